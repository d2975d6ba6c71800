// C ABI (include/lorann.h) and host orchestration of LoRANN's query phase on one MI355X (gfx950).
//
// Kernel sequence of one batch, all on the index's stream, no host synchronisation in between:
//   project (fp64 matrix cores) -> quantize -> centroid dissimilarities (fp64 matrix cores) -> select w
//   clusters (+ bucket histogram) -> scan -> scatter pairs into cluster buckets -> first int8 product +
//   re-quantization (int8 matrix cores, per cluster) -> int8 scores + exact top-m -> exact re-rank + top-k.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/lorann.h"
#include "common.hpp"
#include "gemm_f64.hpp"
#include "rerank.hpp"
#include "rerank_group.hpp"
#include "route.hpp"
#include "score_mfma.hpp"
#include "screen.hpp"
#include "select_exact.hpp"
#include "select_query.hpp"
#include "small_batch.hpp"
#include "screen_fused.hpp"
#include "stage_a.hpp"

using namespace lorann;

// Workspace of lorann_search_noalloc: one fixed region per GPU, part of the loaded code object (every GPU the
// library runs on holds it until the process ends).  In host code this name is only a stand-in for the symbol:
// the device address comes from hipGetSymbolAddress (scratch_of_device below) and only that pointer is ever
// passed to kernels.
static __device__ __align__(256) unsigned char scratch[LORANN_NOALLOC_SCRATCH_BYTES];

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                                      \
    do {                                                                                                   \
        hipError_t e_ = (expr);                                                                            \
        if (e_ != hipSuccess)                                                                              \
            return fail(e_ == hipErrorOutOfMemory ? LORANN_E_NOMEM : LORANN_E_DEVICE, "%s failed: %s", #expr, \
                        hipGetErrorString(e_));                                                            \
    } while (0)

bool is_device_ptr(const void* p) {
    hipPointerAttribute_t at;
    hipError_t e = hipPointerGetAttributes(&at, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();   // plain host memory: clear the sticky error
        return false;
    }
    return at.type == hipMemoryTypeDevice || at.type == hipMemoryTypeManaged;
}

// A fixed region of device memory that buffers are carved from, one after the other (no allocation).
struct Arena {
    unsigned char* base = nullptr;
    size_t cap = 0, used = 0;
};

// Device buffer that grows on demand and is freed with its owner - or, given an arena, a slice of it.
struct DevBuf {
    void* p = nullptr;
    size_t cap = 0;
    int reserve(size_t bytes, Arena* arena = nullptr) {
        if (arena) {
            const size_t at = (arena->used + 255) & ~(size_t)255;
            arena->used = at + bytes;
            if (arena->used > arena->cap) return LORANN_E_UNSUPPORTED;     // the caller reports the total
            p = arena->base + at; cap = bytes;
            return LORANN_OK;
        }
        if (bytes <= cap) return LORANN_OK;
        if (p) { (void)hipFree(p); p = nullptr; cap = 0; }
        size_t want = bytes + bytes / 8 + 256;
        hipError_t e = hipMalloc(&p, want);
        if (e != hipSuccess) { (void)hipGetLastError(); p = nullptr; return fail(LORANN_E_NOMEM, "hipMalloc of %zu bytes failed: %s", want, hipGetErrorString(e)); }
        cap = want;
        return LORANN_OK;
    }
    void release() { if (p) (void)hipFree(p); p = nullptr; cap = 0; }
    template <typename T> T* as() const { return reinterpret_cast<T*>(p); }
};

// Device buffers of one search in flight, sized for one chunk of queries, grown on demand.
struct Workspace {
    DevBuf qproj, qbf, q8, dx, gscore, sel, count, rank_in_bucket, qrank, qorder, qorder2, off0, base_tab, bucket_off, tile_off, unit_off, slot_of_pos, pos_of_slot, Z, sigma, rho0, cand;
    DevBuf tau, n_kept, fb_list, pmax, voff, qkey, u_row, u_mask, u_pos, u_count, rdist, rcid, rccount;
    DevBuf smin, thr, hit_val, hit_grp, hit_cnt;      // screening without the matrix of approximate values
    hipStream_t stream = nullptr;          // lanes >= 1: created on first use, default priority
    hipEvent_t fork = nullptr, join = nullptr;
    hipEvent_t gather_done = nullptr;      // recorded after this lane's latest re-rank gather
    Arena* arena = nullptr;                // set: every buffer is a slice of this fixed region, nothing is allocated or freed
    int64_t last_ngroups = 0;              // groups of the latest grouped re-rank on this workspace (0: none)
    void release() {
        if (arena) return;
        DevBuf* bufs[] = {&qproj, &qbf, &q8, &dx, &gscore, &sel, &count, &rank_in_bucket, &qrank, &qorder, &qorder2, &off0, &base_tab, &bucket_off, &tile_off,
                          &unit_off, &slot_of_pos, &pos_of_slot, &Z, &sigma, &rho0, &cand, &tau, &n_kept, &fb_list, &pmax, &voff, &qkey, &u_row, &u_mask, &u_pos, &u_count, &rdist, &rcid, &rccount};
        for (DevBuf* b : bufs) b->release();
        if (fork) (void)hipEventDestroy(fork);
        if (gather_done) (void)hipEventDestroy(gather_done);
        if (join) (void)hipEventDestroy(join);
        if (stream) (void)hipStreamDestroy(stream);
        fork = join = gather_done = nullptr; stream = nullptr;
    }
};

enum KernelId { K_PROJECT, K_QUANTIZE, K_CENTROID, K_CENTROID_BF16, K_SELECT_W, K_BUCKET_COUNT, K_SCAN, K_SCATTER, K_STAGE_A, K_PAIR_MAX, K_SELECT_QUERY, K_SELECT_M, K_ORDER, K_UNION, K_RERANK, K_TOPK, K_CAND_SCORES, K_COUNT };
const char* const kKernelNames[K_COUNT] = {"project_f64", "quantize_rows", "centroid_dissim_f64", "centroid_screen_bf16", "select_clusters",
                                            "bucket_count", "scan_buckets", "scatter_pairs", "stage_a_i8", "pair_max_i8", "select_query", "score_select_exact",
                                            "order_queries", "group_union", "rerank", "topk", "candidate_scores"};

struct EventPair { hipEvent_t a, b; int kid; };

// Device address of `scratch` on each GPU (every GPU holds its own copy at its own address), looked up once per
// device with that device current.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

int scratch_of_device(int dev, void** out) {
    if (dev < 0 || dev >= kMaxDevices) return fail(LORANN_E_UNSUPPORTED, "device %d is beyond the %d devices the library keeps a scratch pointer for", dev, kMaxDevices);
    if (!g_scratch_ptr[dev]) {
        int cur = -1;
        HIP_TRY(hipGetDevice(&cur));
        if (cur != dev) return fail(LORANN_E_INVAL, "device %d must be current to look up its scratch region (current: %d)", dev, cur);
        void* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return LORANN_OK;
}

}  // namespace

struct lorann_index {
    int32_t metric = 0, d = 0, dp = 0, r = 0, r_pad = 0, L = 0;
    int64_t n = 0;
    hipStream_t stream = nullptr;
    // index data (device)
    float* centroids = nullptr;     // [L][dp]
    double* cent_sqnorm = nullptr;  // [L] (Euclidean)
    float* cent_nrm_f32 = nullptr;  // [L] (Euclidean) the same norms rounded to float, for the approximate scores
    __bf16* cent_bf16 = nullptr;    // [L][dp] centroids rounded to bfloat16
    float mu_max = 0.0f;            // >= max_l |mu_l|_2 (rounded up)
    float dmu_max = 0.0f;           // >= max_l |mu_l - bfloat16(mu_l)|_2 (rounded up)
    float nrm_max = 0.0f;           // >= max_l |mu_l|_2^2 (Euclidean)
    float* Pt = nullptr;            // [dp][d] transposed projection, or NULL
    int8_t* A = nullptr;            // [L][r][dp]
    int8_t* Bp = nullptr;           // [n][r_pad] codes padded with zeros to r_pad bytes
    float *sA = nullptr, *sB = nullptr;
    float* sA_cols = nullptr;       // [L][r] column-wise quantization: step size of every column of A_c (else NULL)
    float* sB_pts = nullptr;        // [n]    ... and of every point's code
    float* A_first = nullptr;       // [L][r] mixed-precision decomposition: unquantized first row of every A_c (else NULL)
    float* B_first = nullptr;       // [n]    ... and of every B_c (one value per point)
    int64_t* off = nullptr;         // [L+1]
    float* corpus = nullptr;        // [n][d]
    _Float16* corpus_h = nullptr;   // [n][d] binary16 copy, made when the half-precision re-rank is first selected
    int32_t rerank_mode = LORANN_RERANK_F32;
    int64_t* ids = nullptr;         // [n] or NULL
    float* sqnorm = nullptr;        // [n] (Euclidean)
    // One workspace per lane.  Lane 0 runs on `stream` (lorann_search, lorann_search_async, lorann_search_stages);
    // the other lanes run on streams of their own, so that batches on different lanes overlap on the GPU.
    Workspace ws[LORANN_LANES];
    int device = 0;                 // the GPU that holds the index
    Workspace ws_fixed;             // lorann_search_noalloc: buffers carved from that GPU's fixed scratch region
    Arena fixed_arena;
    hipEvent_t last_gather = nullptr;   // gather_done of the lane that enqueued the latest gather (owned by that lane)
    int32_t gather_turns = 1;       // the re-rank gathers of different lanes run one after the other
    int32_t force_exact = 0;        // 1: score + select with the per-query kernel only (verification)
    int32_t screen_mode = 0;        // LORANN_SCREEN_AUTO / _MATRIX / _DIGEST
    DevBuf stage_q, stage_ids, stage_dists;   // staging when the caller passes host memory
    DevBuf fb_total;                // while profiling asynchronous searches: device-side sum of the fallback counts
    bool fb_total_live = false;
    // profiling
    bool prof_on = false;
    int prof_only = -1;             // >= 0: record only this kernel (keeps the event overhead out of a timed run)
    std::vector<EventPair> ev_used, ev_free;
    double prof_ms[K_COUNT] = {0};
    int64_t prof_launches[K_COUNT] = {0};
    int64_t prof_fallback_queries = 0;   // queries finished by the exact per-query kernel while profiling
};

namespace {

void free_all(lorann_index* ix) {
    void* ptrs[] = {ix->centroids, ix->cent_sqnorm, ix->cent_nrm_f32, ix->cent_bf16, ix->Pt, ix->A, ix->Bp, ix->sA, ix->sB, ix->sA_cols, ix->sB_pts, ix->A_first, ix->B_first, ix->off, ix->corpus, ix->corpus_h, ix->ids, ix->sqnorm};
    for (void* p : ptrs) if (p) (void)hipFree(p);
    for (Workspace& w : ix->ws) w.release();
    DevBuf* bufs[] = {&ix->stage_q, &ix->stage_ids, &ix->stage_dists, &ix->fb_total};
    for (DevBuf* b : bufs) b->release();
    for (auto& e : ix->ev_used) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    for (auto& e : ix->ev_free) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    delete ix;
}

template <typename T>
int dev_copy(T** dst, const T* src, size_t count) {
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(dst), std::max<size_t>(count, 1) * sizeof(T)));
    if (count) HIP_TRY(hipMemcpy(*dst, src, count * sizeof(T), hipMemcpyDefault));
    return LORANN_OK;
}

__global__ void k_pad_codes(const int8_t* __restrict__ B, int8_t* __restrict__ Bp, int64_t n, int r, int r_pad) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n * r_pad) return;
    const int64_t row = t / r_pad;
    const int j = (int)(t - row * r_pad);
    Bp[t] = j < r ? B[row * r + j] : (int8_t)0;
}

struct Prof {
    lorann_index* ix;
    hipStream_t st;
    int idx = -1;
    Prof(lorann_index* ix_, int kid, hipStream_t st_) : ix(ix_), st(st_) {
        if (!ix->prof_on || (ix->prof_only >= 0 && ix->prof_only != kid)) return;
        EventPair ep;
        if (!ix->ev_free.empty()) { ep = ix->ev_free.back(); ix->ev_free.pop_back(); }
        else if (hipEventCreate(&ep.a) != hipSuccess || hipEventCreate(&ep.b) != hipSuccess) return;
        ep.kid = kid;
        ix->ev_used.push_back(ep);
        idx = (int)ix->ev_used.size() - 1;
        (void)hipEventRecord(ep.a, st);
    }
    ~Prof() { if (idx >= 0) (void)hipEventRecord(ix->ev_used[idx].b, st); }
};

void prof_collect(lorann_index* ix) {   // the stream has been synchronised
    for (auto& e : ix->ev_used) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, e.a, e.b) == hipSuccess) { ix->prof_ms[e.kid] += ms; ix->prof_launches[e.kid] += 1; }
        ix->ev_free.push_back(e);
    }
    ix->ev_used.clear();
}

// Brings the profile totals up to date with everything enqueued so far (asynchronous searches leave their events
// and their fallback counts pending).
int sync_all(lorann_index* ix);

int prof_settle(lorann_index* ix) {
    { const int rc = sync_all(ix); if (rc) return rc; }
    prof_collect(ix);
    if (ix->fb_total_live) {
        int32_t fb = 0;
        HIP_TRY(hipMemcpy(&fb, ix->fb_total.p, 4, hipMemcpyDeviceToHost));
        ix->prof_fallback_queries += fb;
        ix->fb_total_live = false;
    }
    return LORANN_OK;
}

int next_pow2(int v) { int p = 1; while (p < v) p <<= 1; return p; }

constexpr int kSmallPathQueries = 64;   // batches up to this size take the query-major path
constexpr int kNZ = 2;                 // 32-pair tiles per scoring unit
constexpr int kUnitPairs = 32 * kNZ;
constexpr int kChunkTiles = 16;       // 32-point tiles per scoring work item
constexpr int ilog2_exact(int v) { return v == 1 ? 0 : 1 + ilog2_exact(v / 2); }
constexpr int kUnitShift = ilog2_exact(kUnitPairs), kChunkShift = ilog2_exact(32 * kChunkTiles);
static_assert((1 << kUnitShift) == kUnitPairs && (1 << kChunkShift) == 32 * kChunkTiles, "work items are powers of two");
// which shape the pair-maxima kernel takes: at most 16 pairs per cluster on average -> one wavefront streams a cluster
inline bool pair_max_streams(int64_t npairs, int L) { return npairs <= (int64_t)16 * L; }

// S7 on the int8 matrix cores: the best score of every (query, cluster) pair.  With y_off / y (verification) the
// instantiation that also stores every accumulator is launched instead.
void launch_pair_max(lorann_index* ix, Workspace& ws, hipStream_t s, int64_t npairs, const int64_t* y_off, int32_t* y, bool small = false) {
    const int L = small ? (int)npairs : ix->L;       // small batches: every pair is a cluster of its own
    const bool l2 = ix->metric == LORANN_L2, mixed = ix->A_first != nullptr;
    const int ks = ix->r_pad / 32;
    ScoreArgs sc;
    sc.Bp = ix->Bp; sc.Z = ws.Z.as<int8_t>(); sc.sigma = ws.sigma.as<float>(); sc.off = ix->off;
    sc.bucket_off = ws.bucket_off.as<int32_t>(); sc.unit_off = ws.unit_off.as<int32_t>();
    sc.sqnorm = l2 ? ix->sqnorm : nullptr; sc.pt_scale = ix->sB_pts; sc.pt_first = ix->B_first; sc.rho0 = mixed ? ws.rho0.as<float>() : nullptr; sc.pmax = ws.pmax.as<uint32_t>(); sc.L = L; sc.chunk_tiles = kChunkTiles;
    sc.slot_of_pos = ws.slot_of_pos.as<int32_t>(); sc.y_off = y_off; sc.y = y;
    sc.voff = small ? ws.voff.as<int64_t>() : nullptr;
    // few pairs per cluster: the kernel streams the codes of the touched clusters, one wavefront per cluster
    const bool stream = small || pair_max_streams(npairs, L);
    const dim3 gs((unsigned)((L + 3) / 4)), gp(2048);   // persistent shape: 8192 wavefronts stride over the work items
#define LAUNCH_PM4(KS_, L2_, COLS_, MIX_, DUMP_)                                                                      \
    do {                                                                                                             \
        if (stream) hipLaunchKernelGGL((k_pair_max<1, KS_, L2_, 8 / KS_, true, 4, COLS_, MIX_, DUMP_>), gs, dim3(256), 0, s, sc); \
        else hipLaunchKernelGGL((k_pair_max<kNZ, KS_, L2_, 4, false, 4, COLS_, MIX_, DUMP_>), gp, dim3(256), 0, s, sc); \
    } while (0)
#define LAUNCH_PM3(KS_, L2_, DUMP_)                                                                                   \
    do {                                                                                                             \
        if (mixed) LAUNCH_PM4(KS_, L2_, true, true, DUMP_);                                                          \
        else if (ix->sB_pts) LAUNCH_PM4(KS_, L2_, true, false, DUMP_);                                               \
        else LAUNCH_PM4(KS_, L2_, false, false, DUMP_);                                                              \
    } while (0)
#define LAUNCH_PM(KS_, L2_) do { if (y) LAUNCH_PM3(KS_, L2_, true); else LAUNCH_PM3(KS_, L2_, false); } while (0)
    if (ks == 1) { if (l2) LAUNCH_PM(1, true); else LAUNCH_PM(1, false); }
    else         { if (l2) LAUNCH_PM(2, true); else LAUNCH_PM(2, false); }
#undef LAUNCH_PM
#undef LAUNCH_PM3
#undef LAUNCH_PM4
}

// What one batch will run, decided before anything is enqueued.
struct ChunkPlan {
    bool mixed, screen, fused_quant, big_matrix, lds_hist, grouped;
    bool small;         // query-major path of small batches (no bucketing)
    bool digest;        // screening from subset minima and hit lists: the matrix of approximate values is never written
    int group_q;        // queries per re-rank group (0: rows too long to share)
    int nbb;            // blocks of the bucket-count kernel
    int64_t ngroups;
};

ChunkPlan plan_chunk(const lorann_index* ix, int64_t nq, int w, int m) {
    ChunkPlan pl;
    const int L = ix->L;
    pl.mixed = ix->A_first != nullptr;      // Sec. 4.2: first component of q' and of every r stay in float
    // Routing by screening (approximate scores on the bf16 matrix cores, exact evaluation of a short list) unless
    // verification asks for the plain route or the row of values does not fit the registers of a block.
    pl.screen = !ix->force_exact && L <= 16384;
    // With a projection and routing by screening: the projection also writes the bfloat16 copy of q', the selection
    // kernel also quantizes its query and clears the batch's counters - one pass over the queries less.
    pl.fused_quant = pl.screen && ix->Pt != nullptr && !pl.mixed;
    // an approximate-score matrix beyond the caches (256 MB) is streamed: written and read once, nothing of it is worth keeping
    pl.big_matrix = pl.screen && L > 4096 && (int64_t)nq * L * 4 > (int64_t(256) << 20);
    // Many queries x many clusters: the matrix would be written and read once through HBM; two passes of the product
    // that keep only digests are cheaper (measured at L = 16384: from about 5000 queries on; below, the 8 x ceil(nq/512)
    // blocks of a pass leave most CUs idle).  Needs the query operand resident in registers (d' of 128, 192 or 256) and enough
    // centroid tiles for every run of the second grid dimension.
    const bool digest_ok = pl.screen && (ix->dp == 128 || ix->dp == 192 || ix->dp == 256) && L >= 128 * kFusedSplits && w <= kFusedSubsets / 2;
    pl.digest = digest_ok && (ix->screen_mode == LORANN_SCREEN_DIGEST || (ix->screen_mode == LORANN_SCREEN_AUTO && nq >= 6144 && L >= 4096));
    if (pl.digest) pl.big_matrix = false;
    pl.lds_hist = (size_t)L * 8 <= 64 * 1024;
    pl.nbb = (int)((nq + kBucketQueries - 1) / kBucketQueries);
    pl.group_q = rerank_group_size(ix->d);
    pl.grouped = ix->rerank_mode != LORANN_RERANK_NONE && m <= 512 && !ix->force_exact && pl.group_q > 0;
    // A few dozen queries: hardly two pairs share a cluster, so the pairs stay in slot order and every launch that only
    // serves the bucketing is left out (per-cluster step sizes only).
    pl.small = nq <= kSmallPathQueries && pl.screen && !pl.mixed && ix->sA_cols == nullptr && ix->rerank_mode != LORANN_RERANK_NONE;
    // (small batches: a group per query - nothing to share, and the union and the gather of a group are latency chains)
    pl.ngroups = !pl.grouped ? 0 : pl.small ? nq : (nq + pl.group_q - 1) / pl.group_q;
    return pl;
}

// Every device buffer of one batch.  All of them are reserved here, before the first launch, so that a workspace
// that cannot hold the batch is refused while nothing has been enqueued yet.
int reserve_workspace(const lorann_index* ix, Workspace& ws, const ChunkPlan& pl, int64_t nq, int w, int m) {
    const int L = ix->L, dp = ix->dp, r_pad = ix->r_pad;
    const size_t npairs = (size_t)nq * w, q = (size_t)nq;
    Arena* ar = ws.arena;
    if (ar) ar->used = 0;
    struct Want { DevBuf* b; size_t bytes; bool on; };
    const size_t gm = (size_t)pl.group_q * m;
    const bool no_rerank = ix->rerank_mode == LORANN_RERANK_NONE;
    const Want wants[] = {
        {&ws.qproj, q * dp * 4, true}, {&ws.q8, q * dp, true}, {&ws.dx, q * 4, true}, {&ws.gscore, q * L * 4, true},
        {&ws.sel, npairs * 4, true},
        {&ws.count, (size_t)(2 * L + 1) * 4, true},   // [L] pair counters, [L] nearest-cluster counters, fallback-list counter
        {&ws.rank_in_bucket, npairs * 4, true}, {&ws.qrank, q * 4, true}, {&ws.qorder, q * 4, true}, {&ws.qorder2, q * 4, true},
        {&ws.off0, (size_t)L * 4, true}, {&ws.pmax, npairs * 4, true}, {&ws.bucket_off, (size_t)(L + 1) * 4, true},
        {&ws.tile_off, (size_t)(L + 1) * 4, true}, {&ws.unit_off, (size_t)(L + 1) * 4, true},
        {&ws.slot_of_pos, npairs * 4, true}, {&ws.pos_of_slot, npairs * 4, true}, {&ws.Z, npairs * r_pad, true},
        {&ws.sigma, npairs * 4, true}, {&ws.rho0, npairs * 4, pl.mixed}, {&ws.cand, q * m * 4, true},
        {&ws.qbf, q * dp * 2, pl.screen}, {&ws.voff, npairs * 16, pl.small}, {&ws.base_tab, (size_t)2 * pl.nbb * L * 4, pl.lds_hist},
        {&ws.tau, q * 4, !ix->force_exact}, {&ws.n_kept, q * 4, !ix->force_exact}, {&ws.fb_list, q * 4, !ix->force_exact},
        {&ws.qkey, q * 4, !ix->force_exact},
        {&ws.u_row, (size_t)pl.ngroups * gm * 4, pl.grouped}, {&ws.u_mask, (size_t)pl.ngroups * gm * 2, pl.grouped},
        {&ws.u_pos, (size_t)pl.ngroups * gm * pl.group_q * 2, pl.grouped}, {&ws.u_count, (size_t)pl.ngroups * 4, pl.grouped},
        {&ws.rdist, q * m * 4, pl.grouped || no_rerank}, {&ws.rcid, q * m * 8, pl.grouped || no_rerank},
        {&ws.rccount, q * 4, pl.grouped || no_rerank || pl.small},      // (small batches: also the tickets of the one-launch re-rank)
        {&ws.smin, q * kFusedSubsets * 4, pl.digest}, {&ws.thr, q * 4, pl.digest},
        {&ws.hit_val, q * kFusedLists * kFusedCap * 64, pl.digest}, {&ws.hit_grp, q * kFusedLists * kFusedCap * 4, pl.digest},
        {&ws.hit_cnt, q * kFusedLists * 4, pl.digest},
    };
    bool fits = true;
    for (const Want& wt : wants) {
        if (!wt.on) continue;
        const int rc = wt.b->reserve(wt.bytes, ar);
        if (rc == LORANN_OK) continue;
        if (!ar) return rc;
        fits = false;           // keep adding up: the message states the whole requirement
    }
    if (!fits)
        return fail(LORANN_E_UNSUPPORTED, "this search needs %zu bytes of workspace, the fixed scratch region holds %zu (nq = %lld, w = %d, m = %d)",
                    ar->used, ar->cap, (long long)nq, w, m);
    return LORANN_OK;
}

// One batch of at most `chunk` queries, device pointers only.
int search_chunk(lorann_index* ix, Workspace& ws, hipStream_t s, const float* dQ, int64_t nq, int k, int w, int m, int64_t* d_ids,
                 float* d_dists, const lorann_stages* st, int64_t q_base, int32_t* fb_total) {
    const int L = ix->L, dp = ix->dp, d = ix->d, r_pad = ix->r_pad;
    const int64_t npairs = nq * w;
    const ChunkPlan pl = plan_chunk(ix, nq, w, m);
    { const int rc = reserve_workspace(ix, ws, pl, nq, w, m); if (rc) return rc; }
    const bool mixed = pl.mixed;

    const float* qp = dQ;   // projected queries
    const bool fused_quant = pl.fused_quant;
    __bf16* proj_bf = fused_quant ? ws.qbf.as<__bf16>() : nullptr;
    if (ix->Pt) {
        Prof p(ix, K_PROJECT, s);
        const int pvec = (d % 4 == 0 && (reinterpret_cast<uintptr_t>(dQ) & 15u) == 0 && (reinterpret_cast<uintptr_t>(ix->Pt) & 15u) == 0) ? 1 : 0;
        if (nq <= 32)      // a handful of queries: one wavefront per (query, column)
            hipLaunchKernelGGL(k_project_small<1>, dim3((unsigned)((dp + 3) / 4), (unsigned)nq), dim3(256), 0, s, dQ, ix->Pt, ws.qproj.as<float>(), (int)nq, dp, d, proj_bf);
        else if (nq <= kSmallBatch)
            hipLaunchKernelGGL(k_project_small<kSmallM>, dim3((unsigned)((dp + 3) / 4), (unsigned)((nq + kSmallM - 1) / kSmallM)), dim3(256), 0, s, dQ, ix->Pt, ws.qproj.as<float>(), (int)nq, dp, d, proj_bf);
        else {
            // tall tiles for as many whole rounds of the 256 CUs as the batch holds, the rest by whichever height suits it
            const int nbx = (dp + 63) / 64;
            const int64_t round_rows = (int64_t)64 * std::max(1, 256 / nbx);
            const int64_t rows64_full = (nq / round_rows) * round_rows, rem = nq - rows64_full;
            const bool rem_small = rem > 0 && gemm_pick_bm(rem, dp) == 32;
            const int64_t rows64 = rem_small ? rows64_full : nq;
            const int n64 = (int)((rows64 + 63) / 64) * nbx;
            const int n32 = rem_small ? (int)((rem + 31) / 32) * nbx : 0;
            hipLaunchKernelGGL(k_gemm_nt_f64_two_heights<EPI_PLAIN>, dim3((unsigned)(n64 + n32)), dim3(256), 0, s, dQ, ix->Pt, ws.qproj.as<float>(), (const double*)nullptr,
                               (int)nq, dp, d, pvec, proj_bf, n64, (int)rows64);
        }
        qp = ws.qproj.as<float>();
    }
    const bool screen = pl.screen;
    if (!fused_quant) {
        Prof p(ix, K_QUANTIZE, s);
        hipLaunchKernelGGL(k_quantize_rows, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, qp, ws.q8.as<int8_t>(), ws.dx.as<float>(), (int)nq, dp,
                           ws.count.as<int32_t>(), 2 * L + 1, screen ? ws.qbf.as<__bf16>() : (__bf16*)nullptr, mixed ? 1 : 0);
    }
    const bool big_matrix = pl.big_matrix;
    if (screen) {
        if (pl.digest) {
            Prof p(ix, K_CENTROID_BF16, s);
            ScreenPassArgs pa;
            pa.Q = ws.qbf.as<__bf16>(); pa.C = ix->cent_bf16; pa.nrm = ix->metric == LORANN_L2 ? ix->cent_nrm_f32 : nullptr;
            pa.nq = (int)nq; pa.L = L; pa.tiles_per_split = ((L + 63) / 64 + kFusedSplits - 1) / kFusedSplits;
            pa.smin = ws.smin.as<float>(); pa.thr = ws.thr.as<float>(); pa.hit_val = ws.hit_val.as<float>();
            pa.hit_grp = ws.hit_grp.as<int32_t>(); pa.hit_cnt = ws.hit_cnt.as<int32_t>();
            const bool l2 = ix->metric == LORANN_L2;
#define LAUNCH_SP(KS_, L2_, EMIT_, W_) hipLaunchKernelGGL((k_screen_pass<KS_, L2_, EMIT_, W_>), dim3((unsigned)((nq + 64 * W_ - 1) / (64 * W_)), kFusedSplits), dim3(64 * W_), (size_t)2 * (KS_ == 16 ? 64 * 512 : 64 * (32 * KS_ + 16) + 256), s, pa)
#define LAUNCH_SP2(EMIT_, W_) do { if (dp == 128) { if (l2) LAUNCH_SP(8, true, EMIT_, W_); else LAUNCH_SP(8, false, EMIT_, W_); } \
                               else if (dp == 192) { if (l2) LAUNCH_SP(12, true, EMIT_, W_); else LAUNCH_SP(12, false, EMIT_, W_); } \
                               else { if (l2) LAUNCH_SP(16, true, EMIT_, W_); else LAUNCH_SP(16, false, EMIT_, W_); } } while (0)
            // blocks of 512 queries when they fill the 256 CUs at least once, else of 256 (twice the blocks)
            const bool wide = ((nq + 511) / 512) * kFusedSplits >= 256;
            if (wide) LAUNCH_SP2(false, 8); else LAUNCH_SP2(false, 4);
            hipLaunchKernelGGL(k_screen_threshold, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, ws.smin.as<float>(), qp, (int)nq, dp, w, l2, ix->mu_max, ix->dmu_max,
                               l2 ? ix->nrm_max : 0.0f, ws.thr.as<float>());
            if (wide) LAUNCH_SP2(true, 8); else LAUNCH_SP2(true, 4);
#undef LAUNCH_SP2
#undef LAUNCH_SP
        } else {
            Prof p(ix, K_CENTROID_BF16, s);
            const int64_t blocks2 = (int64_t)((L + 127) / 128) * ((nq + 127) / 128);
            const int ti = blocks2 >= 256 ? 2 : 1;          // tiny problems: twice the blocks of half the height
            const dim3 grid((unsigned)((L + 127) / 128), (unsigned)((nq + 64 * ti - 1) / (64 * ti)));
            const float* nrm = ix->metric == LORANN_L2 ? ix->cent_nrm_f32 : nullptr;
#define LAUNCH_CB(L2_, TI_, NT_) hipLaunchKernelGGL((k_centroid_bf16<L2_, TI_, NT_>), grid, dim3(256), 0, s, ws.qbf.as<__bf16>(), ix->cent_bf16, ws.gscore.as<float>(), nrm, (int)nq, L, dp)
            if (big_matrix) { if (ix->metric == LORANN_L2) LAUNCH_CB(true, 2, true); else LAUNCH_CB(false, 2, true); }
            else if (ix->metric == LORANN_L2) { if (ti == 2) LAUNCH_CB(true, 2, false); else LAUNCH_CB(true, 1, false); }
            else { if (ti == 2) LAUNCH_CB(false, 2, false); else LAUNCH_CB(false, 1, false); }
#undef LAUNCH_CB
        }
        {
            Prof p(ix, K_SELECT_W, s);
            ScreenArgs sa;
            sa.ghat = ws.gscore.as<float>(); sa.qp = qp; sa.centroids = ix->centroids;
            sa.cent_sqnorm = ix->metric == LORANN_L2 ? ix->cent_sqnorm : nullptr; sa.sel = ws.sel.as<int32_t>();
            sa.L = L; sa.dp = dp; sa.w = w; sa.mu_max = ix->mu_max; sa.dmu_max = ix->dmu_max; sa.nrm_max = ix->metric == LORANN_L2 ? ix->nrm_max : 0.0f;
            sa.q8 = fused_quant ? ws.q8.as<int8_t>() : nullptr; sa.dx = ws.dx.as<float>();
            sa.zero = fused_quant ? ws.count.as<int32_t>() : nullptr; sa.nzero = 2 * L + 1;
            const size_t lds = (size_t)dp * 4;
            sa.thr = ws.thr.as<float>(); sa.hit_val = ws.hit_val.as<float>(); sa.hit_grp = ws.hit_grp.as<int32_t>(); sa.hit_cnt = ws.hit_cnt.as<int32_t>();
            sa.nlist = kFusedLists; sa.cap = kFusedCap;
            if (pl.digest) hipLaunchKernelGGL((k_select_clusters_screen<1, false, true>), dim3((unsigned)nq), dim3(256), lds, s, sa);
            else if (L <= 1024) hipLaunchKernelGGL(k_select_clusters_screen_wave<16>, dim3((unsigned)((nq + 3) / 4)), dim3(256), 4 * lds, s, sa, (int)nq);
            else if (L <= 2048) hipLaunchKernelGGL(k_select_clusters_screen_wave<32>, dim3((unsigned)((nq + 3) / 4)), dim3(256), 4 * lds, s, sa, (int)nq);
            else if (L <= 4096) hipLaunchKernelGGL(k_select_clusters_screen<16>, dim3((unsigned)nq), dim3(256), lds, s, sa);
            else if (big_matrix) hipLaunchKernelGGL((k_select_clusters_screen<64, true>), dim3((unsigned)nq), dim3(256), lds, s, sa);
            else hipLaunchKernelGGL(k_select_clusters_screen<64>, dim3((unsigned)nq), dim3(256), lds, s, sa);
        }
    } else {
    {
        Prof p(ix, K_CENTROID, s);
        const bool big = gemm_pick_bm(nq, L) == 64;
        const int cvec = (dp % 4 == 0 && (reinterpret_cast<uintptr_t>(qp) & 15u) == 0 && (reinterpret_cast<uintptr_t>(ix->centroids) & 15u) == 0) ? 1 : 0;
        const dim3 grid((L + 63) / 64, (unsigned)(big ? (nq + 63) / 64 : (nq + 31) / 32));
        float* gs = ws.gscore.as<float>();
        if (ix->metric == LORANN_L2) {
            if (big) hipLaunchKernelGGL((k_gemm_nt_f64<EPI_L2, 64>), grid, dim3(256), 0, s, qp, ix->centroids, gs, (const double*)ix->cent_sqnorm, (int)nq, L, dp, cvec);
            else hipLaunchKernelGGL((k_gemm_nt_f64<EPI_L2, 32>), grid, dim3(256), 0, s, qp, ix->centroids, gs, (const double*)ix->cent_sqnorm, (int)nq, L, dp, cvec);
        } else {
            if (big) hipLaunchKernelGGL((k_gemm_nt_f64<EPI_NEG, 64>), grid, dim3(256), 0, s, qp, ix->centroids, gs, (const double*)nullptr, (int)nq, L, dp, cvec);
            else hipLaunchKernelGGL((k_gemm_nt_f64<EPI_NEG, 32>), grid, dim3(256), 0, s, qp, ix->centroids, gs, (const double*)nullptr, (int)nq, L, dp, cvec);
        }
    }
    {
        Prof p(ix, K_SELECT_W, s);
        if (L <= 1024)
            hipLaunchKernelGGL(k_select_clusters_wave<16>, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, ws.gscore.as<float>(), (int)nq, L, w, ws.sel.as<int32_t>());
        else if (L <= 4096)
            hipLaunchKernelGGL(k_select_clusters_wave<64>, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, ws.gscore.as<float>(), (int)nq, L, w, ws.sel.as<int32_t>());
        else if (L <= 8192)
            hipLaunchKernelGGL(k_select_clusters_regs<32>, dim3((unsigned)nq), dim3(256), 0, s, ws.gscore.as<float>(), L, w, ws.sel.as<int32_t>());
        else if (L <= 16384)
            hipLaunchKernelGGL(k_select_clusters_regs<64>, dim3((unsigned)nq), dim3(256), 0, s, ws.gscore.as<float>(), L, w, ws.sel.as<int32_t>());
        else
            hipLaunchKernelGGL(k_select_clusters, dim3((unsigned)nq), dim3(256), 0, s, ws.gscore.as<float>(), L, w, ws.sel.as<int32_t>());
    }
    }
    if (pl.small) {        // small batches: the A stage pair by pair, pairs stay in slot order
        Prof p(ix, K_STAGE_A, s);
        SmallArgs sm;
        sm.q8 = ws.q8.as<int8_t>(); sm.dx = ws.dx.as<float>(); sm.A = ix->A; sm.sA = ix->sA; sm.sB = ix->sB; sm.off = ix->off; sm.r = ix->r; sm.r_pad = r_pad;
        sm.Z = ws.Z.as<int8_t>(); sm.sigma = ws.sigma.as<float>(); sm.pmax = ws.pmax.as<uint32_t>(); sm.pos_of_slot = ws.pos_of_slot.as<int32_t>();
        sm.slot_of_pos = ws.slot_of_pos.as<int32_t>(); sm.voff = ws.voff.as<int64_t>(); sm.qorder = ws.qorder.as<int32_t>(); sm.done = ws.rccount.as<int32_t>();
        const int ppw = r_pad <= 32 ? 2 : 1;
        hipLaunchKernelGGL(k_small_stage_a, dim3((unsigned)((npairs + 4 * ppw - 1) / (4 * ppw))), dim3(256), 0, s, sm, ws.sel.as<int32_t>(), (int)nq, w, dp);
    } else {
    const bool lds_hist = pl.lds_hist;
    const int nbb = pl.nbb;
    int32_t* base_tab = lds_hist ? ws.base_tab.as<int32_t>() : nullptr;
    int32_t* base0_tab = lds_hist ? base_tab + (size_t)nbb * L : nullptr;
    {
        Prof p(ix, K_BUCKET_COUNT, s);
        int32_t* cnt = ws.count.as<int32_t>();
        if (lds_hist)
            hipLaunchKernelGGL(k_bucket_count, dim3((unsigned)nbb), dim3(1024), (size_t)L * 8, s, ws.sel.as<int32_t>(), (int)nq, w, L, cnt, cnt + L,
                               ws.rank_in_bucket.as<int32_t>(), ws.qrank.as<int32_t>(), base_tab, base0_tab);
        else
            hipLaunchKernelGGL(k_bucket_count_global, dim3((unsigned)((npairs + 255) / 256)), dim3(256), 0, s, ws.sel.as<int32_t>(), npairs, w, cnt, cnt + L,
                               ws.rank_in_bucket.as<int32_t>(), ws.qrank.as<int32_t>());
    }
    const bool fused_scan = L <= 1024;       // the scatter kernel scans the counters itself
    if (!fused_scan) {
        Prof p(ix, K_SCAN, s);
        hipLaunchKernelGGL(k_scan_buckets, dim3((unsigned)((L + 1023) / 1024)), dim3(1024), 0, s, ws.count.as<int32_t>(), ws.count.as<int32_t>() + L, ix->off, L, kUnitShift, kChunkShift, ws.bucket_off.as<int32_t>(),
                           ws.tile_off.as<int32_t>(), ws.unit_off.as<int32_t>(), ws.off0.as<int32_t>());
    }
    {
        Prof p(ix, K_SCATTER, s);
        ScanArgs sc;
        sc.count = ws.count.as<int32_t>(); sc.count0 = ws.count.as<int32_t>() + L; sc.off = ix->off; sc.unit_shift = kUnitShift; sc.chunk_shift = kChunkShift;
        sc.tile_off = ws.tile_off.as<int32_t>(); sc.unit_off = ws.unit_off.as<int32_t>();
        if (fused_scan)
            hipLaunchKernelGGL(k_scatter_pairs<true>, dim3((unsigned)((npairs + 255) / 256)), dim3(256), 0, s, ws.sel.as<int32_t>(), npairs, w, L, ws.bucket_off.as<int32_t>(),
                               ws.rank_in_bucket.as<int32_t>(), ws.off0.as<int32_t>(), ws.qrank.as<int32_t>(), base_tab, base0_tab, ws.slot_of_pos.as<int32_t>(),
                               ws.pos_of_slot.as<int32_t>(), ws.pmax.as<uint32_t>(), ws.qorder.as<int32_t>(), sc);
        else
            hipLaunchKernelGGL(k_scatter_pairs<false>, dim3((unsigned)((npairs + 255) / 256)), dim3(256), 0, s, ws.sel.as<int32_t>(), npairs, w, L, ws.bucket_off.as<int32_t>(),
                               ws.rank_in_bucket.as<int32_t>(), ws.off0.as<int32_t>(), ws.qrank.as<int32_t>(), base_tab, base0_tab, ws.slot_of_pos.as<int32_t>(),
                               ws.pos_of_slot.as<int32_t>(), ws.pmax.as<uint32_t>(), ws.qorder.as<int32_t>(), sc);
    }
    {
        Prof p(ix, K_STAGE_A, s);
        // four tiles of 16 pairs per wavefront, dealt from the list of all clusters' tiles (at most npairs / 16 + L of them)
        const int tpw = 4;
        const dim3 grid((unsigned)((npairs / 16 + L + 4 * tpw - 1) / (4 * tpw)));
#define LAUNCH_SA(RT_, RES_)                                                                                   \
    do {                                                                                                       \
        if (ix->sA_cols) hipLaunchKernelGGL((k_stage_a<RT_, RES_, true>), grid, dim3(256), 0, s, ws.q8.as<int8_t>(), ws.dx.as<float>(), ix->A, ix->sA_cols, ix->sB, \
                                            ws.bucket_off.as<int32_t>(), ws.tile_off.as<int32_t>(), tpw, (int)(npairs / 16 + L / 2), ws.slot_of_pos.as<int32_t>(), L, dp, ix->r, w, ws.Z.as<int8_t>(), ws.sigma.as<float>(), \
                                            qp, (const float*)ix->A_first, mixed ? ws.rho0.as<float>() : (float*)nullptr); \
        else hipLaunchKernelGGL((k_stage_a<RT_, RES_, false>), grid, dim3(256), 0, s, ws.q8.as<int8_t>(), ws.dx.as<float>(), ix->A, ix->sA, ix->sB, \
                                ws.bucket_off.as<int32_t>(), ws.tile_off.as<int32_t>(), tpw, (int)(npairs / 16 + L / 2), ws.slot_of_pos.as<int32_t>(), L, dp, ix->r, w, ws.Z.as<int8_t>(), ws.sigma.as<float>(), \
                                (const float*)nullptr, (const float*)nullptr, (float*)nullptr); \
    } while (0)
        if (r_pad == 32) { if (dp <= 256) LAUNCH_SA(2, true); else LAUNCH_SA(2, false); }
        else { if (dp <= 256) LAUNCH_SA(4, true); else LAUNCH_SA(4, false); }
#undef LAUNCH_SA
    }
    }
    // Scores + candidate selection.  Batched path: pair maxima (MFMA) -> per-query walk over the few clusters whose maximum reaches the running m-th best score; the exact per-query kernel finishes what the batched path cannot.
    const int kGroupQ = pl.group_q;
    const bool grouped = pl.grouped;
    SelectArgs sa_;
    sa_.qlist = nullptr; sa_.qcount = nullptr; sa_.fb_total = nullptr; sa_.sel = ws.sel.as<int32_t>(); sa_.pos_of_slot = ws.pos_of_slot.as<int32_t>();
    sa_.Z = ws.Z.as<int8_t>(); sa_.sigma = ws.sigma.as<float>(); sa_.Bp = ix->Bp; sa_.off = ix->off;
    sa_.sqnorm = ix->metric == LORANN_L2 ? ix->sqnorm : nullptr; sa_.pt_scale = ix->sB_pts; sa_.pt_first = ix->B_first; sa_.rho0 = mixed ? ws.rho0.as<float>() : nullptr; sa_.cand = ws.cand.as<int32_t>(); sa_.w = w; sa_.m = m;
    if (ix->force_exact) {
        Prof p(ix, K_SELECT_M, s);
        const unsigned grid = (unsigned)std::min<int64_t>(nq, 65536);
        if (r_pad == 32) hipLaunchKernelGGL(k_select_exact<2>, dim3(grid), dim3(256), 0, s, sa_, (int)nq);
        else hipLaunchKernelGGL(k_select_exact<4>, dim3(grid), dim3(256), 0, s, sa_, (int)nq);
    } else {
        const bool l2 = ix->metric == LORANN_L2;
        const int ks = r_pad / 32;
        {
            Prof p(ix, K_PAIR_MAX, s);
            launch_pair_max(ix, ws, s, npairs, nullptr, nullptr, pl.small);
        }
        {
            Prof p(ix, K_SELECT_QUERY, s);
            QuerySelectArgs qa;
            qa.sel = ws.sel.as<int32_t>(); qa.pos_of_slot = ws.pos_of_slot.as<int32_t>(); qa.pmax = ws.pmax.as<uint32_t>();
            qa.Z = ws.Z.as<int8_t>(); qa.sigma = ws.sigma.as<float>(); qa.Bp = ix->Bp; qa.off = ix->off; qa.sqnorm = l2 ? ix->sqnorm : nullptr; qa.pt_scale = ix->sB_pts; qa.pt_first = ix->B_first; qa.rho0 = mixed ? ws.rho0.as<float>() : nullptr;
            qa.cand = ws.cand.as<int32_t>(); qa.tau = ws.tau.as<float>(); qa.n_kept = ws.n_kept.as<int32_t>(); qa.qkey = ws.qkey.as<int32_t>();
            qa.fb_list = ws.fb_list.as<int32_t>(); qa.fb_count = ws.count.as<int32_t>() + 2 * L; qa.qorder = ws.qorder.as<int32_t>(); qa.nq = (int)nq; qa.w = w; qa.m = m; qa.cap = select_query_cap(m);
            const size_t qlds = (size_t)qa.cap * 8;
            qa.run_shift = 6;
            const int64_t round = (int64_t)8 << qa.run_shift;
            const dim3 qgrid((unsigned)(round * ((nq + round - 1) / round)));
            if (pl.small && qa.cap == 2048) {
                if (ks == 1) hipLaunchKernelGGL((k_select_query<2, 2, true>), qgrid, dim3(256), qlds, s, qa);
                else hipLaunchKernelGGL((k_select_query<4, 2, true>), qgrid, dim3(256), qlds, s, qa);
            } else if (pl.small) {
                if (ks == 1) hipLaunchKernelGGL((k_select_query<2, 6, true>), qgrid, dim3(256), qlds, s, qa);
                else hipLaunchKernelGGL((k_select_query<4, 6, true>), qgrid, dim3(256), qlds, s, qa);
            } else if (qa.cap == 2048) {
                if (ks == 1) hipLaunchKernelGGL((k_select_query<2, 2>), qgrid, dim3(256), qlds, s, qa);
                else hipLaunchKernelGGL((k_select_query<4, 2>), qgrid, dim3(256), qlds, s, qa);
            } else {
                if (ks == 1) hipLaunchKernelGGL((k_select_query<2, 6>), qgrid, dim3(256), qlds, s, qa);
                else hipLaunchKernelGGL((k_select_query<4, 6>), qgrid, dim3(256), qlds, s, qa);
            }
        }
        sa_.qlist = ws.fb_list.as<int32_t>(); sa_.qcount = ws.count.as<int32_t>() + 2 * L;
        sa_.fb_total = fb_total;      // asynchronous searches being profiled: the count is added up on the device
        if (!grouped && !pl.small) {  // (the grouped re-rank finishes these queries in the launch that orders the queries; small batches inline)
            Prof p(ix, K_SELECT_M, s);
            const unsigned grid = (unsigned)std::min<int64_t>(nq, 1024);
            if (r_pad == 32) hipLaunchKernelGGL(k_select_exact<2>, dim3(grid), dim3(256), 0, s, sa_, (int)nq);
            else hipLaunchKernelGGL(k_select_exact<4>, dim3(grid), dim3(256), 0, s, sa_, (int)nq);
        }
    }
    const int mp2 = std::max(256, next_pow2(m));
    const bool half_rows = ix->rerank_mode == LORANN_RERANK_F16;
    if (ix->rerank_mode == LORANN_RERANK_NONE) {
        // no re-ranking step: the candidates (m == k here) are the answer, ordered by their estimated scores
        sa_.qlist = nullptr; sa_.qcount = nullptr; sa_.fb_total = nullptr;
        {
            Prof p(ix, K_CAND_SCORES, s);
            const dim3 grid((unsigned)((nq + 3) / 4));
            if (r_pad == 32) hipLaunchKernelGGL(k_candidate_scores<2>, grid, dim3(256), 0, s, sa_, (int)nq, ix->ids, ws.rdist.as<float>(), ws.rcid.as<int64_t>(), ws.rccount.as<int32_t>());
            else hipLaunchKernelGGL(k_candidate_scores<4>, grid, dim3(256), 0, s, sa_, (int)nq, ix->ids, ws.rdist.as<float>(), ws.rcid.as<int64_t>(), ws.rccount.as<int32_t>());
        }
        GroupArgs ga{};
        ga.dist = ws.rdist.as<float>(); ga.cid = ws.rcid.as<int64_t>(); ga.ccount = ws.rccount.as<int32_t>();
        ga.out_ids = d_ids; ga.out_dists = d_dists; ga.nq = (int)nq; ga.d = d; ga.m = m; ga.k = k;
        {
            Prof p(ix, K_TOPK, s);
            if (k <= 64) hipLaunchKernelGGL(k_topk_wave<4>, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, ga);
            else hipLaunchKernelGGL(k_topk, dim3((unsigned)nq), dim3(256), (size_t)mp2 * 12, s, ga, mp2);
        }
    } else if (grouped) {
        // grouped re-rank: neighbours in the visiting order share candidate rows, each distinct row is gathered once
        if (!pl.small) {          // (small batches: no overflow list to finish, and the queries keep their given order)
            Prof p(ix, K_ORDER, s);
            const int fb_blocks = (int)std::min<int64_t>(nq, 1024);
            const dim3 grid((unsigned)(fb_blocks + L));
            if (r_pad == 32) hipLaunchKernelGGL(k_finish_and_order<2>, grid, dim3(256), 0, s, sa_, fb_blocks, ws.qorder.as<int32_t>(), ws.off0.as<int32_t>(), L, (int)nq, ws.qkey.as<int32_t>(), ws.qorder2.as<int32_t>());
            else hipLaunchKernelGGL(k_finish_and_order<4>, grid, dim3(256), 0, s, sa_, fb_blocks, ws.qorder.as<int32_t>(), ws.off0.as<int32_t>(), L, (int)nq, ws.qkey.as<int32_t>(), ws.qorder2.as<int32_t>());
        }
        if (pl.small && nq <= 8 && d % 4 == 0 && d <= 1024 && k <= 64) {
            // a handful of queries: no union (a query's candidates are distinct rows), distances and top-k in one launch
            // (its per-block device-scope fences cost more than the two launches they save from a few hundred blocks on:
            // measured 106 us against 31 us at 64 queries)
            GroupArgs ga{};
            ga.Q = dQ; ga.corpus = half_rows ? (const void*)ix->corpus_h : (const void*)ix->corpus; ga.ids = ix->ids; ga.cand = ws.cand.as<int32_t>();
            ga.dist = ws.rdist.as<float>(); ga.cid = ws.rcid.as<int64_t>(); ga.ccount = ws.rccount.as<int32_t>();
            ga.out_ids = d_ids; ga.out_dists = d_dists; ga.nq = (int)nq; ga.d = d; ga.m = m; ga.k = k;
            ws.last_ngroups = 0;
            const int slices = std::min(16, (m + 7) / 8);
            const int nv = (d / 4 + 63) / 64;
            Prof p(ix, K_RERANK, s);
            const dim3 grid((unsigned)(nq * slices));
#define LAUNCH_SR4(M_, NV_, T_) do { if (m <= 256) hipLaunchKernelGGL((k_small_rerank<M_, NV_, T_, 4>), grid, dim3(256), 0, s, ga, slices, ws.rccount.as<int32_t>()); \
                                     else hipLaunchKernelGGL((k_small_rerank<M_, NV_, T_, 8>), grid, dim3(256), 0, s, ga, slices, ws.rccount.as<int32_t>()); } while (0)
#define LAUNCH_SR3(M_, NV_) do { if (half_rows) LAUNCH_SR4(M_, NV_, _Float16); else LAUNCH_SR4(M_, NV_, float); } while (0)
#define LAUNCH_SR(M_)                                                                                          \
    do {                                                                                                       \
        switch (nv) {                                                                                          \
            case 1: LAUNCH_SR3(M_, 1); break;                                                                  \
            case 2: LAUNCH_SR3(M_, 2); break;                                                                  \
            case 3: LAUNCH_SR3(M_, 3); break;                                                                  \
            default: LAUNCH_SR3(M_, 4); break;                                                                 \
        }                                                                                                      \
    } while (0)
            if (ix->metric == LORANN_IP) LAUNCH_SR(0);
            else if (ix->metric == LORANN_L2) LAUNCH_SR(1);
            else LAUNCH_SR(2);
#undef LAUNCH_SR
#undef LAUNCH_SR3
#undef LAUNCH_SR4
        } else {
        const int64_t ngroups = pl.ngroups;
        const size_t gm = (size_t)kGroupQ * m;
        GroupArgs ga;
        ga.Q = dQ; ga.corpus = half_rows ? (const void*)ix->corpus_h : (const void*)ix->corpus; ga.ids = ix->ids; ga.cand = ws.cand.as<int32_t>(); ga.qorder = pl.small ? ws.qorder.as<int32_t>() : ws.qorder2.as<int32_t>();
        ga.u_row = ws.u_row.as<int32_t>(); ga.u_mask = ws.u_mask.as<uint16_t>(); ga.u_pos = ws.u_pos.as<uint16_t>(); ga.u_count = ws.u_count.as<int32_t>();
        ga.dist = ws.rdist.as<float>(); ga.cid = ws.rcid.as<int64_t>(); ga.ccount = ws.rccount.as<int32_t>();
        ga.out_ids = d_ids; ga.out_dists = d_dists; ga.nq = (int)nq; ga.d = d; ga.m = m; ga.k = k;
        ga.gq = pl.small ? 1 : kGroupQ;
        ga.ht = rerank_group_ht(ga.gq, m);
        ws.last_ngroups = ngroups;
        // enough gather blocks to keep every CU evenly busy: about 2 MiB of rows per block at most
        ga.slices = (int)std::min<int64_t>(16, std::max<int64_t>(1, ((int64_t)gm * d * 4 / 2) / (2 << 20) + 1));
        while ((int64_t)ga.slices * ngroups < 4096 && ga.slices < 16) ++ga.slices;
        {
            Prof p(ix, K_UNION, s);
            hipLaunchKernelGGL(k_group_union<8>, dim3((unsigned)ngroups), dim3(kUnionThreads), (size_t)ga.ht * 6, s, ga);
        }
        // The gathers of different lanes take turns: each alone saturates HBM, so two at once only stretch each other,
        // while the other stages of the other lanes still run beside a gather.
        const bool turns = ix->gather_turns != 0 && !ws.arena;      // (creating the turn's event is an allocation)
        if (turns && ix->last_gather && ix->last_gather != ws.gather_done) HIP_TRY(hipStreamWaitEvent(s, ix->last_gather, 0));
        {
            Prof p(ix, K_RERANK, s);
            const dim3 grid((unsigned)(ngroups * ga.slices));
            const size_t lds = (size_t)kGroupQ * d * 4;
            const int nv = (d % 4 == 0 && d <= 1024) ? (d / 4 + 63) / 64 : 0;
#define LAUNCH_GG3(M_, NV_)                                                                                    \
    do {                                                                                                       \
        if (half_rows) hipLaunchKernelGGL((k_group_gather<M_, NV_, 8, _Float16>), grid, dim3(kGatherThreads), lds, s, ga); \
        else hipLaunchKernelGGL((k_group_gather<M_, NV_, 8, float>), grid, dim3(kGatherThreads), lds, s, ga);   \
    } while (0)
#define LAUNCH_GG(M_)                                                                                          \
    do {                                                                                                       \
        switch (nv) {                                                                                          \
            case 1: LAUNCH_GG3(M_, 1); break;                                                                  \
            case 2: LAUNCH_GG3(M_, 2); break;                                                                  \
            case 3: LAUNCH_GG3(M_, 3); break;                                                                  \
            case 4: LAUNCH_GG3(M_, 4); break;                                                                  \
            default: LAUNCH_GG3(M_, 0); break;                                                                 \
        }                                                                                                      \
    } while (0)
            if (ix->metric == LORANN_IP) LAUNCH_GG(0);
            else if (ix->metric == LORANN_L2) LAUNCH_GG(1);
            else LAUNCH_GG(2);
#undef LAUNCH_GG3
#undef LAUNCH_GG
        }
        if (turns) {
            if (!ws.gather_done) HIP_TRY(hipEventCreateWithFlags(&ws.gather_done, hipEventDisableTiming));
            HIP_TRY(hipEventRecord(ws.gather_done, s));
            ix->last_gather = ws.gather_done;
        }
        {
            Prof p(ix, K_TOPK, s);
            if (k <= 64 && m <= 256) hipLaunchKernelGGL(k_topk_wave<4>, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, ga);
            else if (k <= 64) hipLaunchKernelGGL(k_topk_wave<8>, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, ga);
            else hipLaunchKernelGGL(k_topk, dim3((unsigned)nq), dim3(256), (size_t)mp2 * 12, s, ga, mp2);
        }
        }   // union + gather + top-k
    } else {
        Prof p(ix, K_RERANK, s);
        const size_t lds = (size_t)d * 4 + (size_t)mp2 * 12;
        const int32_t* cand = ws.cand.as<int32_t>();
        const dim3 rgrid((unsigned)(8 * ((nq + 7) / 8)));
#define LAUNCH_RR(M_)                                                                                          \
    do {                                                                                                       \
        if (half_rows) hipLaunchKernelGGL((k_rerank<M_, _Float16>), rgrid, dim3(256), lds, s, dQ, (const _Float16*)ix->corpus_h, ix->ids, cand, ws.qorder.as<int32_t>(), (int)nq, d, m, mp2, k, d_ids, d_dists); \
        else hipLaunchKernelGGL((k_rerank<M_, float>), rgrid, dim3(256), lds, s, dQ, (const float*)ix->corpus, ix->ids, cand, ws.qorder.as<int32_t>(), (int)nq, d, m, mp2, k, d_ids, d_dists); \
    } while (0)
        if (ix->metric == LORANN_IP) LAUNCH_RR(0);
        else if (ix->metric == LORANN_L2) LAUNCH_RR(1);
        else LAUNCH_RR(2);
#undef LAUNCH_RR
    }
    HIP_TRY(hipGetLastError());

    if (st) {   // export intermediate results (verification only; not part of the timed path)
        HIP_TRY(hipStreamSynchronize(s));
        if (st->qproj) HIP_TRY(hipMemcpy(st->qproj + (size_t)q_base * dp, qp, (size_t)nq * dp * 4, hipMemcpyDefault));
        if (st->q8) HIP_TRY(hipMemcpy(st->q8 + (size_t)q_base * dp, ws.q8.p, (size_t)nq * dp, hipMemcpyDefault));
        if (st->dx) HIP_TRY(hipMemcpy(st->dx + q_base, ws.dx.p, (size_t)nq * 4, hipMemcpyDefault));
        if (st->sel) HIP_TRY(hipMemcpy(st->sel + (size_t)q_base * w, ws.sel.p, (size_t)npairs * 4, hipMemcpyDefault));
        if (st->cand_rows) HIP_TRY(hipMemcpy(st->cand_rows + (size_t)q_base * m, ws.cand.p, (size_t)nq * m * 4, hipMemcpyDefault));
        if (st->tau && !ix->force_exact) HIP_TRY(hipMemcpy(st->tau + q_base, ws.tau.p, (size_t)nq * 4, hipMemcpyDefault));
        if (st->n_survivors && !ix->force_exact) HIP_TRY(hipMemcpy(st->n_survivors + q_base, ws.n_kept.p, (size_t)nq * 4, hipMemcpyDefault));
        if (st->z || st->sigma || st->rho0) {   // bucket order -> slot order on the host
            std::vector<int32_t> pos(npairs);
            std::vector<int8_t> Zh((size_t)npairs * r_pad);
            std::vector<float> sg(npairs), r0(npairs, 0.0f);
            if (mixed) HIP_TRY(hipMemcpy(r0.data(), ws.rho0.p, (size_t)npairs * 4, hipMemcpyDeviceToHost));
            HIP_TRY(hipMemcpy(pos.data(), ws.pos_of_slot.p, (size_t)npairs * 4, hipMemcpyDeviceToHost));
            HIP_TRY(hipMemcpy(Zh.data(), ws.Z.p, (size_t)npairs * r_pad, hipMemcpyDeviceToHost));
            HIP_TRY(hipMemcpy(sg.data(), ws.sigma.p, (size_t)npairs * 4, hipMemcpyDeviceToHost));
            std::vector<int8_t> zo((size_t)npairs * ix->r);
            std::vector<float> so(npairs), ro(npairs);
            for (int64_t p = 0; p < npairs; ++p) {
                memcpy(zo.data() + (size_t)p * ix->r, Zh.data() + (size_t)pos[p] * r_pad, (size_t)ix->r);
                so[p] = sg[pos[p]];
                ro[p] = r0[pos[p]];
            }
            if (st->rho0) HIP_TRY(hipMemcpy(st->rho0 + (size_t)q_base * w, ro.data(), ro.size() * 4, hipMemcpyDefault));
            if (st->z) HIP_TRY(hipMemcpy(st->z + (size_t)q_base * w * ix->r, zo.data(), zo.size(), hipMemcpyDefault));
            if (st->sigma) HIP_TRY(hipMemcpy(st->sigma + (size_t)q_base * w, so.data(), so.size() * 4, hipMemcpyDefault));
        }
        if (st->pmax && !ix->force_exact) {   // keys in bucket order -> scores in slot order
            std::vector<int32_t> pos(npairs);
            std::vector<uint32_t> key(npairs);
            HIP_TRY(hipMemcpy(pos.data(), ws.pos_of_slot.p, (size_t)npairs * 4, hipMemcpyDeviceToHost));
            HIP_TRY(hipMemcpy(key.data(), ws.pmax.p, (size_t)npairs * 4, hipMemcpyDeviceToHost));
            std::vector<float> best(npairs);
            for (int64_t p = 0; p < npairs; ++p) {
                const uint32_t kk = key[pos[p]];
                const uint32_t bits = kk == 0u ? 0xff800000u /* no point: -inf */ : (kk & 0x80000000u) ? (kk & 0x7fffffffu) : ~kk;
                memcpy(&best[p], &bits, 4);
            }
            HIP_TRY(hipMemcpy(st->pmax + (size_t)q_base * w, best.data(), best.size() * 4, hipMemcpyDefault));
        }
        if (st->y && st->y_off) {
            // the caller's offsets may live on the host: stage the slice of this chunk on the device
            std::vector<int64_t> yo(npairs + 1);
            HIP_TRY(hipMemcpy(yo.data(), st->y_off + (size_t)q_base * w, (size_t)(npairs + 1) * 8, hipMemcpyDefault));
            const int64_t y0 = yo[0], y1 = yo[npairs];
            for (auto& v : yo) v -= y0;
            int64_t* d_yo = nullptr; int32_t* d_y = nullptr;
            HIP_TRY(hipMalloc((void**)&d_yo, (size_t)(npairs + 1) * 8));
            hipError_t e = hipMalloc((void**)&d_y, std::max<size_t>((size_t)(y1 - y0), 1) * 4);
            if (e != hipSuccess) { (void)hipFree(d_yo); return fail(LORANN_E_NOMEM, "hipMalloc for the score dump failed"); }
            (void)hipMemcpy(d_yo, yo.data(), (size_t)(npairs + 1) * 8, hipMemcpyHostToDevice);
            // batched selection: the accumulators come from the matrix-core kernel itself (its storing instantiation,
            // same launch shape as the timed one); exact selection forced: from the point-by-point kernel
            if (!ix->force_exact) launch_pair_max(ix, ws, s, npairs, d_yo, d_y, pl.small);
            else if (r_pad == 32) hipLaunchKernelGGL(k_dump_pair_scores<2>, dim3((unsigned)npairs), dim3(256), 0, s, ws.sel.as<int32_t>(), ws.pos_of_slot.as<int32_t>(), ws.Z.as<int8_t>(), ix->Bp, ix->off, d_yo, d_y);
            else hipLaunchKernelGGL(k_dump_pair_scores<4>, dim3((unsigned)npairs), dim3(256), 0, s, ws.sel.as<int32_t>(), ws.pos_of_slot.as<int32_t>(), ws.Z.as<int8_t>(), ix->Bp, ix->off, d_yo, d_y);
            e = hipStreamSynchronize(s);
            if (e == hipSuccess) e = hipMemcpy(st->y + y0, d_y, (size_t)(y1 - y0) * 4, hipMemcpyDefault);
            (void)hipFree(d_yo); (void)hipFree(d_y);
            if (e != hipSuccess) return fail(LORANN_E_DEVICE, "score dump failed: %s", hipGetErrorString(e));
        }
    }
    return LORANN_OK;
}

// The stream a lane runs on; lanes >= 1 get theirs (and the two events that tie them to the index's stream) on
// first use.
int lane_stream(lorann_index* ix, int lane, hipStream_t* out) {
    if (lane == 0) { *out = ix->stream; return LORANN_OK; }
    Workspace& ws = ix->ws[lane];
    if (!ws.stream) {
        HIP_TRY(hipStreamCreateWithFlags(&ws.stream, hipStreamNonBlocking));
        HIP_TRY(hipEventCreateWithFlags(&ws.fork, hipEventDisableTiming));
        HIP_TRY(hipEventCreateWithFlags(&ws.join, hipEventDisableTiming));
    }
    *out = ws.stream;
    return LORANN_OK;
}

// Host wait for everything enqueued on the index's stream and on every lane.
int sync_all(lorann_index* ix) {
    HIP_TRY(hipStreamSynchronize(ix->stream));
    for (int l = 1; l < LORANN_LANES; ++l)
        if (ix->ws[l].stream) HIP_TRY(hipStreamSynchronize(ix->ws[l].stream));
    return LORANN_OK;
}

// fixed = the non-allocating variant: lane 0's stream, buffers from the GPU's fixed scratch region, no allocation of
// any kind (device memory, events, streams) and no host wait.
int search_impl(lorann_index* ix, const float* queries, int64_t nq, int32_t k, int32_t w, int32_t m, int64_t* out_ids,
                float* out_dists, const lorann_stages* st, bool async = false, int lane = 0, bool fixed = false) {
    if (!ix) return fail(LORANN_E_INVAL, "index is NULL");
    if (fixed && ix->prof_on) return fail(LORANN_E_INVAL, "lorann_search_noalloc cannot run while profiling is enabled (profiling creates events)");
    if (lane < 0 || lane >= LORANN_LANES) return fail(LORANN_E_INVAL, "lane = %d is outside 0..%d", lane, LORANN_LANES - 1);
    if (nq < 0) return fail(LORANN_E_INVAL, "nq = %lld is negative", (long long)nq);
    if (ix->rerank_mode == LORANN_RERANK_NONE && k >= 1 && m >= k) m = k;    // the candidates are the answer
    if (k < 1 || m < 1 || k > m) return fail(LORANN_E_INVAL, "need 1 <= k <= m (k = %d, m = %d)", k, m);
    if (w < 1 || w > ix->L) return fail(LORANN_E_INVAL, "need 1 <= w <= L (w = %d, L = %d)", w, ix->L);
    if (w > LORANN_MAX_W) return fail(LORANN_E_UNSUPPORTED, "w = %d exceeds LORANN_MAX_W = %d", w, LORANN_MAX_W);
    if (m > LORANN_MAX_M) return fail(LORANN_E_UNSUPPORTED, "m = %d exceeds LORANN_MAX_M = %d", m, LORANN_MAX_M);
    if (nq == 0) return LORANN_OK;
    if (!queries || !out_ids || !out_dists) return fail(LORANN_E_INVAL, "queries / out_ids / out_dists must not be NULL");
    {
        const int mp2 = std::max(256, next_pow2(m));
        const size_t need = (size_t)ix->d * 4 + (size_t)mp2 * 12;      // the one-query-per-block re-rank must fit
        if (need > 64 * 1024)
            return fail(LORANN_E_UNSUPPORTED, "d = %d with m = %d needs more than 64 KiB of LDS in the re-rank", ix->d, m);
    }
    // batches are processed in chunks that keep nq * w and nq * L within 32-bit indexing and a bounded workspace
    int rc0 = LORANN_OK;
    int64_t chunk = 32768;
    while (chunk > 1 && (chunk * w > (1ll << 30) || chunk * (int64_t)ix->L > (1ll << 31))) chunk >>= 1;

    const bool q_dev = is_device_ptr(queries), i_dev = is_device_ptr(out_ids), d_dev = is_device_ptr(out_dists);
    if (async && !(q_dev && i_dev && d_dev)) return fail(LORANN_E_INVAL, "lorann_search_async / lorann_search_lane need device pointers");
    if (async && ix->prof_on && (rc0 = ix->fb_total.reserve(4))) return rc0;
    Workspace& ws = fixed ? ix->ws_fixed : ix->ws[lane];
    hipStream_t stream = nullptr;
    if ((rc0 = lane_stream(ix, lane, &stream))) return rc0;
    if (fixed) {     // refuse before anything is enqueued if one of the chunks does not fit the scratch region
        int cur = -1;
        HIP_TRY(hipGetDevice(&cur));
        if (cur != ix->device) return fail(LORANN_E_INVAL, "the index lives on device %d, the current device is %d", ix->device, cur);
        const int64_t cn = std::min(chunk, nq);
        const ChunkPlan pl = plan_chunk(ix, cn, w, m);
        if ((rc0 = reserve_workspace(ix, ws, pl, cn, w, m))) return rc0;
    }
    if (lane > 0) {     // the lane starts after what the index's stream holds now (the caller's queries)
        HIP_TRY(hipEventRecord(ws.fork, ix->stream));
        HIP_TRY(hipStreamWaitEvent(stream, ws.fork, 0));
    }
    for (int64_t q0 = 0; q0 < nq; q0 += chunk) {
        const int64_t cn = std::min(chunk, nq - q0);
        const float* dQ = queries + (size_t)q0 * ix->d;
        int64_t* dI = out_ids + (size_t)q0 * k;
        float* dD = out_dists + (size_t)q0 * k;
        int rc;
        if (!q_dev) {
            if ((rc = ix->stage_q.reserve((size_t)cn * ix->d * 4))) return rc;
            HIP_TRY(hipMemcpyAsync(ix->stage_q.p, dQ, (size_t)cn * ix->d * 4, hipMemcpyHostToDevice, stream));
            dQ = ix->stage_q.as<float>();
        }
        if (!i_dev) { if ((rc = ix->stage_ids.reserve((size_t)cn * k * 8))) return rc; dI = ix->stage_ids.as<int64_t>(); }
        if (!d_dev) { if ((rc = ix->stage_dists.reserve((size_t)cn * k * 4))) return rc; dD = ix->stage_dists.as<float>(); }
        int32_t* fb_total = nullptr;
        if (async && ix->prof_on && !ix->force_exact) {
            // while asynchronous searches are profiled, the fallback kernel adds its list length to a device total
            if (!ix->fb_total_live) {      // first use since the totals were read: clear it before any lane adds
                int rcs = sync_all(ix);
                if (rcs) return rcs;
                HIP_TRY(hipMemset(ix->fb_total.p, 0, 4));
                ix->fb_total_live = true;
            }
            fb_total = ix->fb_total.as<int32_t>();
        }
        if ((rc = search_chunk(ix, ws, stream, dQ, cn, k, w, m, dI, dD, st, q0, fb_total))) return rc;
        if (!i_dev) HIP_TRY(hipMemcpyAsync(out_ids + (size_t)q0 * k, dI, (size_t)cn * k * 8, hipMemcpyDeviceToHost, stream));
        if (!d_dev) HIP_TRY(hipMemcpyAsync(out_dists + (size_t)q0 * k, dD, (size_t)cn * k * 4, hipMemcpyDeviceToHost, stream));
        if (async) continue;      // nothing waits here: the results are complete once the stream is
        HIP_TRY(hipStreamSynchronize(stream));
        if (ix->prof_on) {
            {   // events of asynchronous searches on other lanes may still be pending
                int rcs = sync_all(ix);
                if (rcs) return rcs;
            }
            prof_collect(ix);
            if (!ix->force_exact) {
                int32_t fb = 0;
                HIP_TRY(hipMemcpy(&fb, ws.count.as<int32_t>() + 2 * ix->L, 4, hipMemcpyDeviceToHost));
                ix->prof_fallback_queries += fb;
            }
        }
    }
    return LORANN_OK;
}

}  // namespace

extern "C" {

const char* lorann_last_error(void) { return g_err.c_str(); }

int lorann_load_index(lorann_index** out, int32_t metric, int64_t n, int32_t d, int32_t dp, int32_t r, int32_t L,
                      const float* centroids, const float* P, const int8_t* A, const int8_t* B, const float* scale_A,
                      const float* scale_B, const int64_t* cluster_offsets, const float* corpus, const int64_t* ids) {
    if (!out) return fail(LORANN_E_INVAL, "out is NULL");
    if (metric != LORANN_IP && metric != LORANN_L2 && metric != LORANN_COS) return fail(LORANN_E_INVAL, "unknown metric %d", metric);
    if (n < 1 || d < 1 || dp < 1 || r < 1 || L < 1) return fail(LORANN_E_INVAL, "n, d, dp, r, L must be positive");
    if (!centroids || !A || !B || !scale_A || !scale_B || !cluster_offsets || !corpus) return fail(LORANN_E_INVAL, "a required array is NULL");
    if (!P && dp != d) return fail(LORANN_E_INVAL, "P = NULL (identity) requires dp == d (dp = %d, d = %d)", dp, d);
    if (dp % 16 != 0) return fail(LORANN_E_INVAL, "dp = %d must be a multiple of 16", dp);
    if (r % 8 != 0) return fail(LORANN_E_INVAL, "r = %d must be a multiple of 8", r);
    if (dp > LORANN_MAX_DP) return fail(LORANN_E_UNSUPPORTED, "dp = %d exceeds LORANN_MAX_DP = %d", dp, LORANN_MAX_DP);
    if (r > LORANN_MAX_R) return fail(LORANN_E_UNSUPPORTED, "r = %d exceeds LORANN_MAX_R = %d", r, LORANN_MAX_R);
    if (n >= (1ll << 31)) return fail(LORANN_E_UNSUPPORTED, "n = %lld must be below 2^31", (long long)n);

    std::vector<int64_t> off(L + 1);
    if (is_device_ptr(cluster_offsets)) {
        hipError_t e = hipMemcpy(off.data(), cluster_offsets, (size_t)(L + 1) * 8, hipMemcpyDeviceToHost);
        if (e != hipSuccess) { (void)hipGetLastError(); return fail(LORANN_E_DEVICE, "reading cluster_offsets failed: %s", hipGetErrorString(e)); }
    } else {
        memcpy(off.data(), cluster_offsets, (size_t)(L + 1) * 8);
    }
    if (off[0] != 0 || off[L] != n) return fail(LORANN_E_INVAL, "cluster_offsets must start at 0 and end at n");
    for (int c = 0; c < L; ++c)
        if (off[c + 1] < off[c]) return fail(LORANN_E_INVAL, "cluster_offsets decrease at cluster %d", c);

    {   // absmax step sizes are non-negative by construction; the integer-domain score comparisons rely on it
        std::vector<float> sc(2 * (size_t)L);
        const float* src[2] = {scale_A, scale_B};
        for (int t = 0; t < 2; ++t) {
            if (is_device_ptr(src[t])) {
                hipError_t e = hipMemcpy(sc.data() + (size_t)t * L, src[t], (size_t)L * 4, hipMemcpyDeviceToHost);
                if (e != hipSuccess) { (void)hipGetLastError(); return fail(LORANN_E_DEVICE, "reading the scales failed: %s", hipGetErrorString(e)); }
            } else {
                memcpy(sc.data() + (size_t)t * L, src[t], (size_t)L * 4);
            }
        }
        for (size_t i = 0; i < sc.size(); ++i)
            if (!(sc[i] >= 0.0f) || sc[i] > 3.0e38f) return fail(LORANN_E_INVAL, "scale_%c[%zu] must be finite and >= 0", i < (size_t)L ? 'A' : 'B', i % L);
    }

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) { (void)hipGetLastError(); return fail(LORANN_E_DEVICE, "no HIP device"); }

    lorann_index* ix = new (std::nothrow) lorann_index();
    if (!ix) return fail(LORANN_E_NOMEM, "out of host memory");
    {   // set-up of the non-allocating entry point: this GPU's address of the fixed scratch region
        void* sp = nullptr;
        int rcs = LORANN_OK;
        if (hipGetDevice(&ix->device) != hipSuccess) { (void)hipGetLastError(); rcs = fail(LORANN_E_DEVICE, "hipGetDevice failed"); }
        else rcs = scratch_of_device(ix->device, &sp);
        if (rcs != LORANN_OK) { delete ix; return rcs; }
        ix->fixed_arena.base = static_cast<unsigned char*>(sp);
        ix->fixed_arena.cap = LORANN_NOALLOC_SCRATCH_BYTES;
        ix->ws_fixed.arena = &ix->fixed_arena;
    }
    ix->metric = metric; ix->n = n; ix->d = d; ix->dp = dp; ix->r = r; ix->L = L;
    ix->r_pad = r <= 32 ? 32 : 64;
    int rc = LORANN_OK;
    auto body = [&]() -> int {
        int e;
        if ((e = dev_copy(&ix->centroids, centroids, (size_t)L * dp))) return e;
        if ((e = dev_copy(&ix->A, A, (size_t)L * r * dp))) return e;
        if ((e = dev_copy(&ix->sA, scale_A, (size_t)L))) return e;
        if ((e = dev_copy(&ix->sB, scale_B, (size_t)L))) return e;
        if ((e = dev_copy(&ix->off, off.data(), (size_t)L + 1))) return e;
        if ((e = dev_copy(&ix->corpus, corpus, (size_t)n * d))) return e;
        if (ids && (e = dev_copy(&ix->ids, ids, (size_t)n))) return e;
        {   // codes padded to r_pad bytes per point so that every point is one or two aligned 32-byte operands
            int8_t* Braw = nullptr;
            if ((e = dev_copy(&Braw, B, (size_t)n * r))) return e;
            // 32 zero rows follow the last point: the scoring kernel requests whole 32-point tiles
            hipError_t he = hipMalloc((void**)&ix->Bp, (size_t)(n + 32) * ix->r_pad);
            if (he != hipSuccess) { (void)hipFree(Braw); return fail(LORANN_E_NOMEM, "hipMalloc of padded codes failed"); }
            (void)hipMemset(ix->Bp + (size_t)n * ix->r_pad, 0, (size_t)32 * ix->r_pad);
            const int64_t tot = n * ix->r_pad;
            hipLaunchKernelGGL(k_pad_codes, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, 0, Braw, ix->Bp, n, r, ix->r_pad);
            he = hipDeviceSynchronize();
            (void)hipFree(Braw);
            if (he != hipSuccess) return fail(LORANN_E_DEVICE, "padding the codes failed: %s", hipGetErrorString(he));
        }
        if (P) {
            float* Praw = nullptr;
            if ((e = dev_copy(&Praw, P, (size_t)d * dp))) return e;
            hipError_t he = hipMalloc((void**)&ix->Pt, (size_t)d * dp * 4);
            if (he != hipSuccess) { (void)hipFree(Praw); return fail(LORANN_E_NOMEM, "hipMalloc of the projection failed"); }
            const int64_t tot = (int64_t)d * dp;
            hipLaunchKernelGGL(k_transpose, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, 0, Praw, ix->Pt, d, dp);
            he = hipDeviceSynchronize();
            (void)hipFree(Praw);
            if (he != hipSuccess) return fail(LORANN_E_DEVICE, "transposing the projection failed: %s", hipGetErrorString(he));
        }
        {   // centroid norms: |mu_l|^2 enters the Euclidean routing (Sec. 3.1); the largest norm enters the error
            // bound of the approximate centroid scores
            double* nrm = nullptr;
            HIP_TRY(hipMalloc((void**)&nrm, (size_t)L * 8));
            hipLaunchKernelGGL(k_row_sqnorm<double>, dim3((unsigned)((L + 3) / 4)), dim3(256), 0, 0, ix->centroids, nrm, (int64_t)L, dp);
            std::vector<double> h((size_t)L);
            hipError_t he = hipMemcpy(h.data(), nrm, (size_t)L * 8, hipMemcpyDeviceToHost);
            if (he != hipSuccess) { (void)hipFree(nrm); return fail(LORANN_E_DEVICE, "centroid norms failed: %s", hipGetErrorString(he)); }
            double mx = 0.0;
            for (double v : h) mx = std::max(mx, v);          // a NaN norm is ignored here; such rows are garbage anyway
            ix->mu_max = std::nextafter((float)(std::sqrt(mx) * (1.0 + 1e-6)), INFINITY);
            ix->nrm_max = std::nextafter((float)(mx * (1.0 + 1e-6)), INFINITY);
            if (metric == LORANN_L2) {
                ix->cent_sqnorm = nrm;
                std::vector<float> hf((size_t)L);
                for (size_t i = 0; i < hf.size(); ++i) hf[i] = (float)h[i];
                if ((e = dev_copy(&ix->cent_nrm_f32, hf.data(), (size_t)L))) return e;
            } else {
                (void)hipFree(nrm);
            }
            HIP_TRY(hipMalloc((void**)&ix->cent_bf16, (size_t)L * dp * 2));
            const int64_t tot = (int64_t)L * dp;
            hipLaunchKernelGGL(k_to_bf16, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, 0, ix->centroids, ix->cent_bf16, tot);
            // the largest rounding error of a centroid enters the same bound
            double* err = nullptr;
            HIP_TRY(hipMalloc((void**)&err, (size_t)L * 8));
            hipLaunchKernelGGL(k_row_bf16_err, dim3((unsigned)((L + 3) / 4)), dim3(256), 0, 0, ix->centroids, ix->cent_bf16, err, (int64_t)L, dp);
            he = hipMemcpy(h.data(), err, (size_t)L * 8, hipMemcpyDeviceToHost);
            (void)hipFree(err);
            if (he != hipSuccess) return fail(LORANN_E_DEVICE, "centroid rounding errors failed: %s", hipGetErrorString(he));
            double mxe = 0.0;
            for (double v : h) mxe = std::max(mxe, v);
            ix->dmu_max = std::nextafter((float)(std::sqrt(mxe) * (1.0 + 1e-6)), INFINITY);
            HIP_TRY(hipDeviceSynchronize());
        }
        if (metric == LORANN_L2) {   // Sec. 3.1: the norms |c_j|^2 of the corpus rows are precomputed
            HIP_TRY(hipMalloc((void**)&ix->sqnorm, (size_t)n * 4));
            hipLaunchKernelGGL(k_row_sqnorm<float>, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, 0, ix->corpus, ix->sqnorm, n, d);
            HIP_TRY(hipDeviceSynchronize());
        }
        return LORANN_OK;
    };
    rc = body();
    if (rc != LORANN_OK) { std::string keep = g_err; free_all(ix); g_err = keep; return rc; }
    *out = ix;
    return LORANN_OK;
}

// The serialized index: a 64-byte header ("LRNIDX01", metric, d, d', r, L, flags, n) and the arrays of
// lorann_load_index, each at a multiple of 64 bytes.  The file is read into host memory and handed to
// lorann_load_index, which validates it like any other caller's arrays.
int lorann_load_index_file(lorann_index** out, const char* path) {
    if (!out || !path) return fail(LORANN_E_INVAL, "lorann_load_index_file: NULL argument");
    FILE* f = fopen(path, "rb");
    if (!f) return fail(LORANN_E_INVAL, "cannot open index file '%s'", path);
    struct Closer { FILE* f; ~Closer() { fclose(f); } } closer{f};
    unsigned char head[64];
    if (fread(head, 1, sizeof head, f) != sizeof head || memcmp(head, "LRNIDX01", 8) != 0)
        return fail(LORANN_E_INVAL, "'%s' is not a LRNIDX01 index file", path);
    int32_t hv[6];
    int64_t n;
    memcpy(hv, head + 8, sizeof hv);
    memcpy(&n, head + 32, sizeof n);
    const int32_t metric = hv[0], d = hv[1], dp = hv[2], r = hv[3], L = hv[4], flags = hv[5];
    if (n < 1 || d < 1 || dp < 1 || r < 1 || L < 1 || n >= (int64_t(1) << 31) || (flags & ~3))
        return fail(LORANN_E_INVAL, "index file '%s': bad header", path);
    int64_t pos = 64;
    auto read_section = [&](std::vector<unsigned char>& buf, size_t bytes) -> bool {
        const int64_t at = (pos + 63) / 64 * 64;
        if (fseeko(f, (off_t)at, SEEK_SET) != 0) return false;
        try { buf.resize(bytes); } catch (...) { return false; }
        size_t got = 0;
        while (got < bytes) {
            const size_t k = fread(buf.data() + got, 1, std::min<size_t>(bytes - got, (size_t)1 << 28), f);
            if (k == 0) return false;
            got += k;
        }
        pos = at + (int64_t)bytes;
        return true;
    };
    std::vector<unsigned char> off, ids, cent, P, A, B, sA, sB, corpus;
    const bool ok = read_section(off, ((size_t)L + 1) * 8) && (!(flags & 2) || read_section(ids, (size_t)n * 8)) &&
                    read_section(cent, (size_t)L * dp * 4) && (!(flags & 1) || read_section(P, (size_t)d * dp * 4)) &&
                    read_section(A, (size_t)L * r * dp) && read_section(B, (size_t)n * r) && read_section(sA, (size_t)L * 4) &&
                    read_section(sB, (size_t)L * 4) && read_section(corpus, (size_t)n * d * 4);
    if (!ok) return fail(LORANN_E_INVAL, "index file '%s' is truncated (or host memory ran out reading it)", path);
    return lorann_load_index(out, metric, n, d, dp, r, L, reinterpret_cast<const float*>(cent.data()),
                             (flags & 1) ? reinterpret_cast<const float*>(P.data()) : nullptr,
                             reinterpret_cast<const int8_t*>(A.data()), reinterpret_cast<const int8_t*>(B.data()),
                             reinterpret_cast<const float*>(sA.data()), reinterpret_cast<const float*>(sB.data()),
                             reinterpret_cast<const int64_t*>(off.data()), reinterpret_cast<const float*>(corpus.data()),
                             (flags & 2) ? reinterpret_cast<const int64_t*>(ids.data()) : nullptr);
}

void lorann_free_index(lorann_index* ix) {
    if (!ix) return;
    (void)sync_all(ix);
    free_all(ix);
}

int lorann_set_stream(lorann_index* ix, void* hip_stream) {
    if (!ix) return fail(LORANN_E_INVAL, "index is NULL");
    HIP_TRY(hipStreamSynchronize(ix->stream));
    ix->stream = reinterpret_cast<hipStream_t>(hip_stream);
    return LORANN_OK;
}

int lorann_search(lorann_index* ix, const float* queries, int64_t nq, int32_t k, int32_t w, int32_t m, int64_t* out_ids,
                  float* out_dists) {
    return search_impl(ix, queries, nq, k, w, m, out_ids, out_dists, nullptr);
}

int lorann_search_async(lorann_index* ix, const float* queries, int64_t nq, int32_t k, int32_t w, int32_t m, int64_t* out_ids,
                        float* out_dists) {
    return search_impl(ix, queries, nq, k, w, m, out_ids, out_dists, nullptr, true);
}

int lorann_search_lane(lorann_index* ix, int32_t lane, const float* queries, int64_t nq, int32_t k, int32_t w, int32_t m,
                       int64_t* out_ids, float* out_dists) {
    return search_impl(ix, queries, nq, k, w, m, out_ids, out_dists, nullptr, true, lane);
}

int lorann_search_noalloc(lorann_index* ix, const float* queries, int64_t nq, int32_t k, int32_t w, int32_t m,
                          int64_t* out_ids, float* out_dists) {
    return search_impl(ix, queries, nq, k, w, m, out_ids, out_dists, nullptr, true, 0, true);
}

int lorann_lane_join(lorann_index* ix, int32_t lane) {
    if (!ix) return fail(LORANN_E_INVAL, "index is NULL");
    if (lane < 0 || lane >= LORANN_LANES) return fail(LORANN_E_INVAL, "lane = %d is outside 0..%d", lane, LORANN_LANES - 1);
    Workspace& ws = ix->ws[lane];
    if (lane == 0 || !ws.stream) return LORANN_OK;       // lane 0 is the index's stream itself; an unused lane holds nothing
    HIP_TRY(hipEventRecord(ws.join, ws.stream));
    HIP_TRY(hipStreamWaitEvent(ix->stream, ws.join, 0));
    return LORANN_OK;
}

int lorann_set_gather_turns(lorann_index* ix, int32_t on) {
    if (!ix) return fail(LORANN_E_INVAL, "index is NULL");
    { const int rc = sync_all(ix); if (rc) return rc; }
    ix->gather_turns = on != 0;
    ix->last_gather = nullptr;
    return LORANN_OK;
}

int lorann_search_stages(lorann_index* ix, const float* queries, int64_t nq, int32_t k, int32_t w, int32_t m,
                         int64_t* out_ids, float* out_dists, const lorann_stages* st) {
    return search_impl(ix, queries, nq, k, w, m, out_ids, out_dists, st);
}

int lorann_set_column_scales(lorann_index* ix, const float* scale_A_columns, const float* scale_B_points) {
    if (!ix) return fail(LORANN_E_INVAL, "index is NULL");
    if ((scale_A_columns == nullptr) != (scale_B_points == nullptr)) return fail(LORANN_E_INVAL, "give both arrays of step sizes, or NULL for both");
    float *na = nullptr, *nb = nullptr;
    if (scale_A_columns) {
        const size_t cnt[2] = {(size_t)ix->L * ix->r, (size_t)ix->n};
        const float* src[2] = {scale_A_columns, scale_B_points};
        for (int t = 0; t < 2; ++t) {      // step sizes are non-negative and finite, as at load time
            std::vector<float> h(cnt[t]);
            hipError_t e = hipMemcpy(h.data(), src[t], cnt[t] * 4, hipMemcpyDefault);
            if (e != hipSuccess) { (void)hipGetLastError(); return fail(LORANN_E_DEVICE, "reading the step sizes failed: %s", hipGetErrorString(e)); }
            for (size_t i = 0; i < cnt[t]; ++i)
                if (!(h[i] >= 0.0f) || h[i] > 3.0e38f) return fail(LORANN_E_INVAL, "scale_%s[%zu] must be finite and >= 0", t ? "B_points" : "A_columns", i);
        }
        int rc;
        if ((rc = dev_copy(&na, scale_A_columns, cnt[0]))) return rc;
        if ((rc = dev_copy(&nb, scale_B_points, cnt[1]))) { (void)hipFree(na); return rc; }
    }
    { const int rc = sync_all(ix); if (rc) return rc; }   // no search may still be reading the old arrays
    if (ix->sA_cols) (void)hipFree(ix->sA_cols);
    if (ix->sB_pts) (void)hipFree(ix->sB_pts);
    ix->sA_cols = na; ix->sB_pts = nb;
    if (!na) {      // the float first rows belong to the column-wise scheme: they go with it
        if (ix->A_first) (void)hipFree(ix->A_first);
        if (ix->B_first) (void)hipFree(ix->B_first);
        ix->A_first = ix->B_first = nullptr;
    }
    return LORANN_OK;
}

int lorann_set_first_rows(lorann_index* ix, const float* first_row_A, const float* first_row_B) {
    if (!ix) return fail(LORANN_E_INVAL, "index is NULL");
    if ((first_row_A == nullptr) != (first_row_B == nullptr)) return fail(LORANN_E_INVAL, "give both first rows, or NULL for both");
    if (first_row_A && !ix->sA_cols) return fail(LORANN_E_INVAL, "the mixed-precision decomposition needs the column-wise step sizes (lorann_set_column_scales first)");
    float *na = nullptr, *nb = nullptr;
    if (first_row_A) {
        const size_t cnt[2] = {(size_t)ix->L * ix->r, (size_t)ix->n};
        const float* src[2] = {first_row_A, first_row_B};
        for (int t = 0; t < 2; ++t) {
            std::vector<float> h(cnt[t]);
            hipError_t e = hipMemcpy(h.data(), src[t], cnt[t] * 4, hipMemcpyDefault);
            if (e != hipSuccess) { (void)hipGetLastError(); return fail(LORANN_E_DEVICE, "reading the first rows failed: %s", hipGetErrorString(e)); }
            for (size_t i = 0; i < cnt[t]; ++i)
                if (!(std::fabs(h[i]) <= 3.0e38f)) return fail(LORANN_E_INVAL, "first_row_%s[%zu] must be finite", t ? "B" : "A", i);
        }
        int rc;
        if ((rc = dev_copy(&na, first_row_A, cnt[0]))) return rc;
        if ((rc = dev_copy(&nb, first_row_B, cnt[1]))) { (void)hipFree(na); return rc; }
    }
    { const int rc = sync_all(ix); if (rc) return rc; }   // no search may still be reading the old arrays
    if (ix->A_first) (void)hipFree(ix->A_first);
    if (ix->B_first) (void)hipFree(ix->B_first);
    ix->A_first = na; ix->B_first = nb;
    return LORANN_OK;
}

int lorann_set_rerank(lorann_index* ix, int32_t mode) {
    if (!ix) return fail(LORANN_E_INVAL, "index is NULL");
    if (mode != LORANN_RERANK_F32 && mode != LORANN_RERANK_F16 && mode != LORANN_RERANK_NONE) return fail(LORANN_E_INVAL, "unknown re-rank mode %d", mode);
    { const int rc = sync_all(ix); if (rc) return rc; }   // searches in flight keep the mode they were enqueued with
    if (mode == LORANN_RERANK_F16 && !ix->corpus_h) {
        const size_t count = (size_t)ix->n * ix->d;
        _Float16* h = nullptr;
        uint32_t* mx = nullptr;
        HIP_TRY(hipMalloc((void**)&h, count * 2));
        hipError_t e = hipMalloc((void**)&mx, 4);
        if (e == hipSuccess) e = hipMemset(mx, 0, 4);
        uint32_t bits = 0;
        if (e == hipSuccess) {
            const unsigned grid = (unsigned)std::min<size_t>((count + 255) / 256, 16384);
            hipLaunchKernelGGL(k_corpus_to_half, dim3(grid), dim3(256), 0, nullptr, ix->corpus, h, count, mx);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipMemcpy(&bits, mx, 4, hipMemcpyDeviceToHost);
        if (mx) (void)hipFree(mx);
        if (e != hipSuccess) { (void)hipFree(h); (void)hipGetLastError(); return fail(e == hipErrorOutOfMemory ? LORANN_E_NOMEM : LORANN_E_DEVICE, "building the half-precision corpus failed: %s", hipGetErrorString(e)); }
        float mxf; memcpy(&mxf, &bits, 4);
        if (!(mxf <= 65504.0f)) { (void)hipFree(h); return fail(LORANN_E_UNSUPPORTED, "the corpus holds values beyond the binary16 range (largest magnitude %g)", (double)mxf); }
        ix->corpus_h = h;
    }
    ix->rerank_mode = mode;
    return LORANN_OK;
}

int lorann_set_exact_selection(lorann_index* ix, int32_t on) {
    if (!ix) return fail(LORANN_E_INVAL, "index is NULL");
    { const int rc = sync_all(ix); if (rc) return rc; }   // searches in flight keep the path they were enqueued with
    ix->force_exact = on != 0;
    return LORANN_OK;
}

int lorann_set_screen_mode(lorann_index* ix, int32_t mode) {
    if (!ix) return fail(LORANN_E_INVAL, "index is NULL");
    if (mode != LORANN_SCREEN_AUTO && mode != LORANN_SCREEN_MATRIX && mode != LORANN_SCREEN_DIGEST) return fail(LORANN_E_INVAL, "unknown screening mode %d", (int)mode);
    { const int rc = sync_all(ix); if (rc) return rc; }   // searches in flight keep the path they were enqueued with
    ix->screen_mode = mode;
    return LORANN_OK;
}

int lorann_profile_enable(lorann_index* ix, int32_t on) {
    if (!ix) return fail(LORANN_E_INVAL, "index is NULL");
    { const int rc = prof_settle(ix); if (rc) return rc; }
    ix->prof_on = on != 0;
    ix->prof_only = on == 2 ? (int)K_RERANK : on == 3 ? (int)K_PAIR_MAX : -1;
    if (on) { for (int i = 0; i < K_COUNT; ++i) { ix->prof_ms[i] = 0.0; ix->prof_launches[i] = 0; } ix->prof_fallback_queries = 0; }
    return LORANN_OK;
}

int64_t lorann_profile_fallback_queries(lorann_index* ix) {
    if (!ix) return -1;
    if (prof_settle(ix) != LORANN_OK) return -1;
    return ix->prof_fallback_queries;
}

int64_t lorann_profile_gather_rows(lorann_index* ix) {
    if (!ix) return -1;
    if (sync_all(ix) != LORANN_OK) return -1;
    const Workspace& ws = ix->ws[0];
    if (ws.last_ngroups <= 0 || !ws.u_count.p) return -1;
    std::vector<int32_t> h((size_t)ws.last_ngroups);
    if (hipMemcpy(h.data(), ws.u_count.p, h.size() * 4, hipMemcpyDeviceToHost) != hipSuccess) { (void)hipGetLastError(); return -1; }
    int64_t tot = 0;
    for (int32_t v : h) tot += v;
    return tot;
}

int lorann_profile_get(lorann_index* ix, lorann_kernel_time* out, int32_t cap) {
    if (!ix) return fail(LORANN_E_INVAL, "index is NULL");
    if (cap > 0 && !out) return fail(LORANN_E_INVAL, "out is NULL");
    { const int rc = prof_settle(ix); if (rc) return rc; }
    for (int i = 0; i < K_COUNT && i < cap; ++i) {
        memset(out[i].name, 0, sizeof out[i].name);
        strncpy(out[i].name, kKernelNames[i], sizeof out[i].name - 1);
        out[i].ms = ix->prof_ms[i];
        out[i].launches = ix->prof_launches[i];
    }
    return K_COUNT;
}

}  // extern "C"
