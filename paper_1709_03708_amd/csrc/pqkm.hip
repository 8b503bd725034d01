// C ABI of the PQk-means iteration for gfx950: argument validation, workspace carving and
// kernel launches.  Every entry point is declared and documented in include/pqkm.h.
#include "pqkm.h"
#include "pqkm_tuning.h"

#include <hip/hip_runtime.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "pqkm_kernels.h"

// Scratch of pqkm_assign_noalloc: one array per GPU, held from the moment the library is loaded on it until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress, never an address to pass on.
static __device__ __align__(256) unsigned char scratch[PQKM_NOALLOC_SCRATCH_BYTES];

namespace {

using namespace pqkm;

// ------------------------------------------------------------------ options and profiling state
struct Options {
    int assign_kernel = 0;   // 0 auto, 1 generic, 2 tiled
    int scan_variant = 0;    // 0 auto, else a specific instantiation (tuning)
    int hist_kernel = 0;     // 0 auto, 1 global atomics, 2 LDS-privatised owner path, 3 sorted by cluster
    int profile = 0;         // bit 0: bracket scan kernels with events, bit 1: bracket whole assignment steps
    int64_t launch_codes = (int64_t)1 << 26;   // codes per scan launch
    int rounds_per_launch = 1;                 // big scans: rounds of workgroups per kernel launch, 0 = all in one
};
Options g_opt;
std::mutex g_mu;
constexpr int HIST_GROUPS = 64;        // target number of cluster groups of the LDS-privatised histogram (measured best)

// Every entry point reads the process-wide options once, here, and passes the copy down: a call never sees a
// change that another thread makes while it runs.
Options options_snapshot()
{
    std::lock_guard<std::mutex> lk(g_mu);
    return g_opt;
}

struct EventPair { hipEvent_t a, b; };
struct EventLog {
    std::vector<EventPair> pool;    // all events ever created
    size_t used = 0;                // pairs recorded since the last read
    int64_t kernels = 0;            // kernel launches inside those pairs (scan log only)
};
EventLog g_scan_log, g_step_log;    // around the scan kernels of a stretch of codes / around every whole assignment step
// scan kernels launched by this thread since it was last cleared: a stretch of codes is one launch, or one launch
// per round of workgroups
thread_local int64_t t_scan_kernels = 0;

// start of a bracket: takes (or creates) a pair and records its first event; false if none could be had
bool log_begin(EventLog& log, hipStream_t st, EventPair* ev)
{
    {
        std::lock_guard<std::mutex> lk(g_mu);
        if (log.used == log.pool.size()) {
            EventPair e{};
            if (hipEventCreate(&e.a) == hipSuccess && hipEventCreate(&e.b) == hipSuccess) log.pool.push_back(e);
        }
        if (log.used == log.pool.size()) return false;
        *ev = log.pool[log.used++];
    }
    hipEventRecord(ev->a, st);
    return true;
}

pqkm_status log_read(EventLog& log, double* total_ms, int64_t* count)
{
    if (!total_ms || !count) return PQKM_ERR_NULL;
    std::lock_guard<std::mutex> lk(g_mu);
    double tot = 0.0;
    for (size_t i = 0; i < log.used; ++i) {
        if (hipEventSynchronize(log.pool[i].b) != hipSuccess) return PQKM_ERR_DEVICE;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, log.pool[i].a, log.pool[i].b) != hipSuccess) return PQKM_ERR_DEVICE;
        tot += ms;
    }
    *total_ms = tot;
    *count = log.kernels ? log.kernels : (int64_t)log.used;
    log.used = 0;
    log.kernels = 0;
    return PQKM_OK;
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline bool tiled_M(int M) { return M == 4 || M == 8 || M == 16 || M == 32; }

struct Carve {
    size_t img_off, img_bytes, hist_off, hist_bytes, counts_off, counts_bytes, parts_off, parts_bytes, gid_off,
        gid_bytes, gco_off, plan_off, rows_off, gc8_off, plan8_off, sidx_off, seg_off, pool_off, bseg_off, skew_off,
        rank_off, tabt_off, rowoff_off, total;
};

// The regrouped copy of the codes (M = 4 scan) covers one scan launch of at most this many codes.
constexpr int64_t GROUP_CHUNK_MAX = (int64_t)1 << 26;
inline int64_t group_alloc(int64_t n) { return (n + 30) & ~(int64_t)15; }  // regrouped positions for n codes
constexpr int SW_C_MAX = 256 * 16;          // most codes a workgroup of the sliding-window scan takes
inline int64_t sw_alloc(int64_t n) { return ((n + SW_C_MAX - 1) / SW_C_MAX + 1) * SW_C_MAX; }   // whole workgroups of any shape

// Shape of the LDS-privatised histogram pass: KT clusters per workgroup, `groups` cluster groups, S code slices.
struct HistPlan { int KT; int64_t groups; int S; bool cheap; };

HistPlan hist_plan(int64_t N, int M, int K)
{
    HistPlan p{};
    const int kt_max = (HIST_LDS_WORDS / L) / M;           // 128 KB of LDS / (M KB per cluster)
    if (kt_max < 1) return p;
    // about HIST_GROUPS groups (a byte names at most 255), within the LDS budget
    const int hg = HIST_GROUPS;
    int kt = (K + hg - 1) / hg;
    if (kt > kt_max) kt = kt_max;
    p.KT = kt;
    p.groups = ((int64_t)K + p.KT - 1) / p.KT;
    p.S = 1;
    while (p.groups * p.S < 192 && p.S < 16 && N / (2 * p.S) >= 8192) p.S *= 2;
    // every cluster group streams one byte per code: worth it while the groups fit a byte and that stays small
    p.cheap = p.groups <= 255 && (double)p.groups * (double)N <= 2.0e9;
    return p;
}

Carve carve(int64_t N, int M, int K)
{
    Carve c{};
    size_t off = 0;
    c.img_off = off;
    if (tiled_M(M)) {
        int TK = 128 / M;
        size_t ntiles = ((size_t)K + TK - 1) / TK;
        c.img_bytes = ntiles * (size_t)TILE_BYTES;
        // the sliding-window scan of the wide codes tiles the centers 16 at a time (M planes of 16 KB per tile)
        if (M >= 16) {
            const size_t wide = (((size_t)K + 15) / 16) * (size_t)M * 16384;
            if (wide > c.img_bytes) c.img_bytes = wide;
        }
    }
    off += align256(c.img_bytes);
    c.hist_off = off;
    c.hist_bytes = (size_t)K * M * L * sizeof(uint32_t);
    off += align256(c.hist_bytes);
    c.counts_off = off;
    c.counts_bytes = (size_t)K * sizeof(uint32_t);
    off += align256(c.counts_bytes);
    c.parts_off = off;
    HistPlan hp = hist_plan(N, M, K);
    c.parts_bytes = (hp.KT >= 1 && hp.S > 1) ? (size_t)hp.S * align256(c.hist_bytes) : 0;
    off += c.parts_bytes;
    c.gid_off = off;
    c.gid_bytes = (hp.KT >= 1 && hp.groups <= 255) ? (size_t)N : 0;
    off += align256(c.gid_bytes);
    c.gco_off = c.plan_off = c.rows_off = off;
    if (M == 4) {
        c.rows_off = off;                    // second copy of the tile images, read by the half-plane scan's epilogue
        off += align256(c.img_bytes);
        const int64_t na = group_alloc(N < GROUP_CHUNK_MAX ? N : GROUP_CHUNK_MAX);
        c.gco_off = off;
        off += align256((size_t)na * sizeof(uint2));
        c.plan_off = off;
        off += align256(sizeof(GroupPlan));
        // records the scan files by cluster group for the histogram (one scan launch, owner-path sizes only): every
        // scan workgroup owns as many records as it has code positions (at most 4096); one segment per (group, workgroup)
        c.pool_off = c.bseg_off = off;
        if (hp.KT >= 1 && hp.groups <= 255 && N <= GROUP_CHUNK_MAX - 16384) {
            c.pool_off = off;
            off += align256((size_t)(na + 4096) * sizeof(uint2));
            c.bseg_off = off;
            off += align256((size_t)hp.groups * (size_t)(na / 2048 + 2) * sizeof(uint2));
        }
    }
    // sorted-path histogram: code indices sorted by cluster (u32), cluster sizes, starts and cursors
    c.sidx_off = c.seg_off = off;
    if (N <= (int64_t)0xffffffff) {
        c.sidx_off = off;
        off += align256((size_t)N * sizeof(uint32_t));
        c.seg_off = off;
        off += 3 * align256(((size_t)K + 1) * sizeof(uint32_t));
        c.rank_off = off;                    // every code's rank inside its cluster, left by the scan (pqkm_fit)
        off += align256((size_t)N * sizeof(uint32_t));
    }
    c.gc8_off = c.plan8_off = off;
    if (M == 8) {
        const int64_t na = group_alloc(N < GROUP_CHUNK_MAX ? N : GROUP_CHUNK_MAX);
        c.gc8_off = off;
        off += align256((size_t)na * sizeof(uint4));
        c.plan8_off = off;
        off += align256(sizeof(GroupPlan8));
    }
    // table-built tiles (M = 4): transposed tables with a row of +inf, row offsets of the centers per tile and plane
    c.tabt_off = c.rowoff_off = off;
    if (M == 4) {
        c.tabt_off = off;
        off += align256(((size_t)M * L + 1) * L * sizeof(float));
        c.rowoff_off = off;
        off += align256((((size_t)K + 31) / 32) * 128 * sizeof(uint32_t));
    }
    // subcode words of the sliding-window scan (M = 16, 32): M/4 + 1 words per code position of one launch
    c.skew_off = off;
    if (M == 16 || M == 32) {
        const int64_t na = sw_alloc(N < GROUP_CHUNK_MAX ? N : GROUP_CHUNK_MAX);
        off += align256((size_t)na * (size_t)(M / 4 + 1) * sizeof(uint32_t));
    }
    c.total = off;
    return c;
}

bool shape_ok(int64_t N, int M, int K) { return N >= 0 && K >= 1 && M >= 1 && M <= 64; }

pqkm_status check_device()
{
    static thread_local int checked_dev = -1;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PQKM_ERR_DEVICE;
    if (dev == checked_dev) return PQKM_OK;
    hipDeviceProp_t p;
    if (hipGetDeviceProperties(&p, dev) != hipSuccess) return PQKM_ERR_DEVICE;
    if (strncmp(p.gcnArchName, "gfx950", 6) != 0) return PQKM_ERR_DEVICE;
    checked_dev = dev;
    return PQKM_OK;
}

// Device address of `scratch` on the current device: asked of the runtime once per device (each GPU holds its own
// copy at its own address) and kept.
constexpr int SCRATCH_MAX_DEVICES = 64;
void* g_scratch_ptr[SCRATCH_MAX_DEVICES];
std::mutex g_scratch_mu;

pqkm_status scratch_of_current_device(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= SCRATCH_MAX_DEVICES) return PQKM_ERR_DEVICE;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PQKM_ERR_DEVICE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return PQKM_OK;
}

pqkm_status launched()
{
    return hipGetLastError() == hipSuccess ? PQKM_OK : PQKM_ERR_DEVICE;
}

pqkm_status check_workspace(const void* ws, size_t bytes, size_t need)
{
    if (need == 0) return PQKM_OK;
    if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || bytes < need) return PQKM_ERR_WORKSPACE;
    return PQKM_OK;
}

// compute units of the current device (asked once; 256 if the query fails)
int cu_count()
{
    static const int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1)
            v = 256;
        return v;
    }();
    return n;
}

// ------------------------------------------------------------------ scan launch
template <int M, int R, int THREADS, bool PF>
void launch_scan(const uint8_t* codes, int64_t N, const float4* img, int ntiles, int32_t* assign, float* dist,
                 hipStream_t st)
{
    using S = ScanShape<M>;
    constexpr int C = (THREADS / S::LPS) * R;
    int64_t nwg = (N + C - 1) / C;
    hipLaunchKernelGGL((assign_scan_kernel<M, R, THREADS, PF>), dim3((unsigned)nwg), dim3(THREADS), 0, st, codes, N,
                       img, ntiles, assign, dist);
}

template <int R, int THREADS>
void launch_scan4s(const uint8_t* codes, int64_t N, const float4* img, int ntiles, int32_t* assign, float* dist,
                   hipStream_t st)
{
    constexpr int C = (THREADS / 4) * R;
    int64_t nwg = (N + C - 1) / C;
    hipLaunchKernelGGL((assign_scan4s_kernel<R, THREADS>), dim3((unsigned)nwg), dim3(THREADS), 0, st, codes, N, img,
                       ntiles, assign, dist);
}

template <int R, int THREADS, int DEPTH, bool BUCKET = false>
void launch_scan4p(const uint8_t* codes, int64_t N, const uint2* gco, const float4* img, const float4* rows,
                   int ntiles, int32_t* assign, float* dist, hipStream_t st, BucketOut bo = BucketOut{},
                   RankOut ro = RankOut{})
{
    constexpr int C = (THREADS / 4) * R;
    int64_t nwg = (N + C - 1) / C;
    hipLaunchKernelGGL((assign_scan4p_kernel<R, THREADS, DEPTH, BUCKET>), dim3((unsigned)nwg), dim3(THREADS), 0, st, codes,
                       N, gco, img, rows, ntiles, assign, dist, bo, ro);
}

template <int M, int R, int THREADS, int DEPTH = 1>
void launch_scan_skew(const uint8_t* codes, int64_t N, const float4* img, int ntiles, int32_t* assign, float* dist,
                      hipStream_t st)
{
    constexpr int C = (THREADS / (128 / M / 4)) * R;
    int64_t nwg = (N + C - 1) / C;
    hipLaunchKernelGGL((assign_scan_skew_kernel<M, R, THREADS, DEPTH>), dim3((unsigned)nwg), dim3(THREADS), 0, st, codes,
                       N, img, ntiles, assign, dist);
}

// tile image layout a scan shape reads: 0 = [m][x][k], 1 = [x][m][k] (subspace-skewed scans), 2 = half planes
// (variant 0, the default for M = 4, regroups the codes and runs the half-plane scan; variant 34 is the
// subspace-skewed scan, which needs no regrouping and is used for few centers or few codes)
inline int variant_layout(int M, int variant)
{
    if (M == 4) {
        if ((variant >= 40 && variant <= 49) || (variant >= 70 && variant <= 99)) return 2;
        return (variant >= 30 && variant <= 39) ? 1 : 0;
    }
    if (M == 8 && ((variant >= 40 && variant <= 49) || (variant >= 70 && variant <= 84))) return 0;   // [m][x][k]
    return variant != 1 ? 1 : 0;  // M = 8, 16, 32: every other shape but 1 (the unskewed tiled scan) is skewed
}

template <int R, int THREADS, int DEPTH>
void launch_scan8p(const uint8_t* codes, int64_t N, const uint4* gc8, const float4* img, int ntiles, int32_t* assign,
                   float* dist, hipStream_t st, RankOut ro = RankOut{}, int rounds_per_launch = 0)
{
    constexpr int C = (THREADS / 4) * R;
    int64_t nwg = (N + C - 1) / C;
    if (gc8 && rounds_per_launch > 0) {
        // regrouped codes, results go to the codes' original positions: any stretch of workgroups can be a launch
        // of its own, and the workgroups of a launch start in step (see launch_scan4q_rounds)
        const int64_t per = (int64_t)rounds_per_launch * cu_count();
        for (int64_t w0 = 0; w0 < nwg; w0 += per) {
            const int64_t cnt = nwg - w0 < per ? nwg - w0 : per;
            hipLaunchKernelGGL((assign_scan8p_kernel<R, THREADS, DEPTH>), dim3((unsigned)cnt), dim3(THREADS), 0, st, codes,
                               N - w0 * C, gc8 + w0 * C, img, ntiles, assign, dist, ro);
            ++t_scan_kernels;
        }
        return;
    }
    hipLaunchKernelGGL((assign_scan8p_kernel<R, THREADS, DEPTH>), dim3((unsigned)nwg), dim3(THREADS), 0, st, codes, N,
                       gc8, img, ntiles, assign, dist, ro);
}

template <int M>
void launch_scan_M(int variant, const uint8_t* codes, int64_t N, const float4* img, const float4* rows, int ntiles,
                   int32_t* assign, float* dist, hipStream_t st);

// Sliding-window scan of the wide codes (variants 50..59): the subcode words of this launch, then the scan.
// Shapes: 512 threads with 16 or 8 codes per lane-slot (4096 or 2048 codes per workgroup, variants 51 and 52) and
// 1024 threads with 6 (3072 codes, variant 53); variant 50 chooses by the number of rounds: a round costs about
// R + 5.5 with 512 threads (R codes' reads per phase, a 64 KB fill worth 4 and two barriers) and, measured, 0.73 of
// the 16-code round with 1024 threads (16.3 ms against 11.9 ms per round at M = 32, K = 1e4).
struct SwShape { int R, threads; };
inline SwShape sw_shape(int variant, int64_t n)
{
    if (variant == 51) return {16, 512};
    if (variant == 52) return {8, 512};
    if (variant == 53) return {6, 1024};
    const int ncu = cu_count();
    static const SwShape cand[] = {{16, 512}, {6, 1024}, {8, 512}};
    static const double round_cost[] = {21.5, 15.7, 13.5};
    SwShape best = cand[0];
    double best_cost = 1e300;
    for (int i = 0; i < 3; ++i) {
        const int64_t C = (int64_t)(cand[i].threads / 2) * cand[i].R;
        const int64_t wgs = (n + C - 1) / C;
        const double cost = (double)((wgs + ncu - 1) / ncu) * round_cost[i];
        if (cost < best_cost) { best_cost = cost; best = cand[i]; }
    }
    return best;
}

template <int M>
pqkm_status launch_scan_sw(int variant, const uint8_t* codes, int64_t N, uint32_t* S, const float4* img, int ntiles16,
                           int32_t* assign, float* dist, hipStream_t st, RankOut ro = RankOut{}, int rounds_per_launch = 0)
{
    const SwShape sh = sw_shape(variant, N);
    const bool wide = sh.threads == 1024;
    const int R = sh.R;
    const int64_t C = (int64_t)(sh.threads / 2) * R;
    const int64_t nwg = (N + C - 1) / C;
    const int64_t n_alloc = nwg * C;
    hipLaunchKernelGGL((code_skew_kernel<M>), dim3((unsigned)((n_alloc + 255) / 256)), dim3(256), 0, st, codes, N, S,
                       n_alloc);
    // kernel launches of rounds_per_launch rounds of workgroups each, so that the workgroups start in step again
    // (see launch_scan4q_rounds)
    const int64_t per = rounds_per_launch > 0 ? (int64_t)rounds_per_launch * cu_count() : nwg;
    for (int64_t w0 = 0; w0 < nwg; w0 += per) {
        const int64_t cnt = nwg - w0 < per ? nwg - w0 : per;
        if (wide)
            hipLaunchKernelGGL((assign_scan_sw_kernel<M, 6, 1024, 2>), dim3((unsigned)cnt), dim3(1024), 0, st, codes, N, S,
                               n_alloc, img, ntiles16, assign, dist, ro, w0);
        else if (R == 8)
            hipLaunchKernelGGL((assign_scan_sw_kernel<M, 8, 512, 3>), dim3((unsigned)cnt), dim3(512), 0, st, codes, N, S,
                               n_alloc, img, ntiles16, assign, dist, ro, w0);
        else
            hipLaunchKernelGGL((assign_scan_sw_kernel<M, 16, 512, 2>), dim3((unsigned)cnt), dim3(512), 0, st, codes, N, S,
                               n_alloc, img, ntiles16, assign, dist, ro, w0);
        ++t_scan_kernels;
    }
    return launched();
}

// M = 4 scans over regrouped codes: variants 70..79

// Codes per lane-slot R of the 512-thread half-plane scan (a workgroup takes 128 R codes, one workgroup per
// compute unit at a time).  The time of a launch is about rounds * (R + 7) with rounds = ceil(workgroups / CUs):
// R codes' reads per tile plus a fill and two barriers worth about 7.  Below a few rounds the rounding decides:
// 1.1e6 codes are 269 workgroups at R = 32, two rounds, but 430 at R = 20, two rounds of 5/8 the length.
int scan4p_codes_per_slot(int64_t n_alloc)
{
    const int ncu = cu_count();
    static const int cand[] = {32, 31, 28, 24, 20, 16};
    int best = 32;
    int64_t best_cost = INT64_MAX;
    for (int R : cand) {
        const int64_t wgs = (n_alloc + 128 * R - 1) / (128 * R);
        const int64_t cost = ((wgs + ncu - 1) / ncu) * (R + 7);
        if (cost < best_cost) { best_cost = cost; best = R; }
    }
    return best;
}

// bo != nullptr: the scan also files (code, center) records by cluster group for the histogram pass (variant 70
// only); *nwg_out receives the number of scan workgroups = the row length of the segment table
void launch_scan_grouped(int variant, const uint2* gco, int64_t n_alloc, const float4* img, const float4* rows,
                         int ntiles, int32_t* assign, float* dist, hipStream_t st, const BucketOut* bo = nullptr,
                         int* nwg_out = nullptr, RankOut ro = RankOut{})
{
    int R = 0;
    switch (variant) {
        case 70: R = scan4p_codes_per_slot(n_alloc); break;
        case 71: R = 28; break;
        case 72: R = 31; break;
        case 73: launch_scan4p<16, 1024, 1>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, BucketOut{}, ro); return;
        case 74: R = 24; break;
        case 75: R = 20; break;
        case 76: R = 16; break;
        default: R = 32; break;      // 77..79
    }
    if (bo) {
        if (nwg_out) *nwg_out = (int)((n_alloc + 128 * R - 1) / (128 * R));
        switch (R) {
            case 16: launch_scan4p<16, 512, 3, true>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, *bo); break;
            case 20: launch_scan4p<20, 512, 3, true>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, *bo); break;
            case 24: launch_scan4p<24, 512, 3, true>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, *bo); break;
            case 28: launch_scan4p<28, 512, 3, true>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, *bo); break;
            case 31: launch_scan4p<31, 512, 3, true>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, *bo); break;
            default: launch_scan4p<32, 512, 3, true>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, *bo); break;
        }
        return;
    }
    switch (R) {
        case 16: launch_scan4p<16, 512, 3>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, BucketOut{}, ro); break;
        case 20: launch_scan4p<20, 512, 3>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, BucketOut{}, ro); break;
        case 24: launch_scan4p<24, 512, 3>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, BucketOut{}, ro); break;
        case 28: launch_scan4p<28, 512, 3>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, BucketOut{}, ro); break;
        case 31: launch_scan4p<31, 512, 3>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, BucketOut{}, ro); break;
        default: launch_scan4p<32, 512, 3>(nullptr, n_alloc, gco, img, rows, ntiles, assign, dist, st, BucketOut{}, ro); break;
    }
}

// M = 4 scan over regrouped codes with two-lane slots (256 R codes per workgroup): variants 80..89
int scan4q_codes_per_slot(int variant, int64_t n_alloc)
{
    // (32 and 30 codes per lane-slot spill registers inside the tile loop: 0.49 and 0.61 of the LDS peak against 0.72)
    switch (variant) {
        case 81: return 26;
        case 82: return 28;
        case 83: return 24;
        case 84: return 16;
        default: break;
    }
    const int ncu = cu_count();
    static const int cand[] = {28, 26, 24, 16};
    int best = 28;
    int64_t best_cost = INT64_MAX;
    for (int R : cand) {
        const int64_t wgs = (n_alloc + 256 * R - 1) / (256 * R);
        const int64_t cost = ((wgs + ncu - 1) / ncu) * (2 * R + 13);      // 512 R clocks of reads per tile, about 3.3k of fill and barriers
        if (cost < best_cost) { best_cost = cost; best = R; }
    }
    return best;
}

template <int R>
void launch_scan4q_rounds(const uint2* gco, int64_t n_alloc, const float4* img, const float4* rows, int ntiles,
                          int32_t* assign, float* dist, hipStream_t st, RankOut ro, int rounds_per_launch)
{
    // The workgroups of a kernel launch start together and walk the tile images in step, so that a tile is fetched
    // from memory once per XCD and then served from its L2; over many rounds of workgroups they drift apart.  With
    // rounds_per_launch > 0 the codes are issued in kernel launches of that many rounds, each starting in step again.
    constexpr int64_t C = 256 * (int64_t)R;
    const int64_t nwg = (n_alloc + C - 1) / C;
    const int64_t per = rounds_per_launch > 0 ? (int64_t)rounds_per_launch * cu_count() : nwg;
    for (int64_t w0 = 0; w0 < nwg; w0 += per) {
        const int64_t cnt = nwg - w0 < per ? nwg - w0 : per;
        hipLaunchKernelGGL((assign_scan4q_kernel<R, 512, 2>), dim3((unsigned)cnt), dim3(512), 0, st, n_alloc - w0 * C,
                           gco + w0 * C, img, rows, ntiles, assign, dist, ro, TileSource{});
        ++t_scan_kernels;
    }
}

void launch_scan_grouped_q(int variant, const uint2* gco, int64_t n_alloc, const float4* img, const float4* rows,
                           int ntiles, int32_t* assign, float* dist, hipStream_t st, RankOut ro, TileSource ts,
                           int rounds_per_launch)
{
    const int R = scan4q_codes_per_slot(variant >= 90 ? variant - 10 : variant, n_alloc);
    const int64_t nwg = (n_alloc + 256 * (int64_t)R - 1) / (256 * (int64_t)R);
    if (ts.tabT) {
        switch (R) {
            case 16:
                hipLaunchKernelGGL((assign_scan4q_kernel<16, 512, 2, true>), dim3((unsigned)nwg), dim3(512), 0, st, n_alloc,
                                   gco, img, rows, ntiles, assign, dist, ro, ts);
                break;
            case 24:
                hipLaunchKernelGGL((assign_scan4q_kernel<24, 512, 2, true>), dim3((unsigned)nwg), dim3(512), 0, st, n_alloc,
                                   gco, img, rows, ntiles, assign, dist, ro, ts);
                break;
            case 26:
                hipLaunchKernelGGL((assign_scan4q_kernel<26, 512, 2, true>), dim3((unsigned)nwg), dim3(512), 0, st, n_alloc,
                                   gco, img, rows, ntiles, assign, dist, ro, ts);
                break;
            default:
                hipLaunchKernelGGL((assign_scan4q_kernel<28, 512, 2, true>), dim3((unsigned)nwg), dim3(512), 0, st, n_alloc,
                                   gco, img, rows, ntiles, assign, dist, ro, ts);
                break;
        }
        return;
    }
    switch (R) {
        case 16: launch_scan4q_rounds<16>(gco, n_alloc, img, rows, ntiles, assign, dist, st, ro, rounds_per_launch); break;
        case 24: launch_scan4q_rounds<24>(gco, n_alloc, img, rows, ntiles, assign, dist, st, ro, rounds_per_launch); break;
        case 26: launch_scan4q_rounds<26>(gco, n_alloc, img, rows, ntiles, assign, dist, st, ro, rounds_per_launch); break;
        default: launch_scan4q_rounds<28>(gco, n_alloc, img, rows, ntiles, assign, dist, st, ro, rounds_per_launch); break;
    }
}

// M = 4, two-lane slots, half tiles loaded straight into LDS (variants 85..89): codes per workgroup
struct Scan4hShape { int R, threads; };
Scan4hShape scan4h_shape(int variant)
{
    switch (variant) {
        case 86: return {12, 1024};
        case 87: return {14, 1024};
        case 88: return {32, 512};
        case 89: return {8, 1024};
        default: return {16, 1024};
    }
}
inline int64_t scan4h_codes_per_workgroup(int variant)
{
    const Scan4hShape sh = scan4h_shape(variant);
    return (int64_t)(sh.threads / 2) * sh.R;
}

template <int R, int THREADS, int DEPTH>
void launch_scan4h_rounds(const uint2* gco, int64_t n_alloc, const float4* img, const float4* rows, int ntiles,
                          int nhalves, int32_t* assign, float* dist, hipStream_t st, RankOut ro, int rounds_per_launch)
{
    // one kernel launch per rounds_per_launch rounds of workgroups (see launch_scan4q_rounds)
    constexpr int64_t C = (THREADS / 2) * (int64_t)R;
    const int64_t nwg = (n_alloc + C - 1) / C;
    const int64_t per = rounds_per_launch > 0 ? (int64_t)rounds_per_launch * cu_count() : nwg;
    for (int64_t w0 = 0; w0 < nwg; w0 += per) {
        const int64_t cnt = nwg - w0 < per ? nwg - w0 : per;
        hipLaunchKernelGGL((assign_scan4h_kernel<R, THREADS, DEPTH>), dim3((unsigned)cnt), dim3(THREADS), 0, st,
                           n_alloc - w0 * C, gco + w0 * C, img, rows, ntiles, nhalves, assign, dist, ro);
        ++t_scan_kernels;
    }
}

void launch_scan_grouped_h(int variant, const uint2* gco, int64_t n_alloc, const float4* img, const float4* rows,
                           int ntiles, int nhalves, int32_t* assign, float* dist, hipStream_t st, RankOut ro,
                           int rounds_per_launch)
{
    switch (variant) {
        case 86: launch_scan4h_rounds<12, 1024, 4>(gco, n_alloc, img, rows, ntiles, nhalves, assign, dist, st, ro, rounds_per_launch); break;
        case 87: launch_scan4h_rounds<14, 1024, 3>(gco, n_alloc, img, rows, ntiles, nhalves, assign, dist, st, ro, rounds_per_launch); break;
        case 88: launch_scan4h_rounds<32, 512, 2>(gco, n_alloc, img, rows, ntiles, nhalves, assign, dist, st, ro, rounds_per_launch); break;
        case 89: launch_scan4h_rounds<8, 1024, 3>(gco, n_alloc, img, rows, ntiles, nhalves, assign, dist, st, ro, rounds_per_launch); break;
        default: launch_scan4h_rounds<16, 1024, 3>(gco, n_alloc, img, rows, ntiles, nhalves, assign, dist, st, ro, rounds_per_launch); break;
    }
}

// The 4096-code shape of the LDS-direct scan, filing (code, center) records by cluster group for the histogram: all
// workgroups in one launch (a segment is named by its workgroup's index in the grid).
void launch_scan4h_bucket(const uint2* gco, int64_t n_alloc, const float4* img, const float4* rows, int ntiles,
                          int nhalves, int32_t* assign, float* dist, hipStream_t st, BucketOut bo, int* nwg_out)
{
    constexpr int64_t C = 512 * 8;
    const int64_t nwg = (n_alloc + C - 1) / C;
    hipLaunchKernelGGL((assign_scan4h_kernel<8, 1024, 3, true>), dim3((unsigned)nwg), dim3(1024), 0, st, n_alloc, gco, img,
                       rows, ntiles, nhalves, assign, dist, RankOut{}, bo);
    ++t_scan_kernels;
    *nwg_out = (int)nwg;
}

// M = 4, many codes: the four-lane scan (variant 70) or one of the shapes of the LDS-direct scan (85..87, 89), by the time
// the rounds of workgroups take.  Clocks per tile and workgroup of C codes, from the measured times: four lanes per
// code 2.30 C + 2065 (the fill of 128 KB between two barriers), LDS-direct 2.45 C + 1064 (two halves).
int choose_scan4_large(int64_t n)
{
    const int ncu = cu_count();
    const int64_t na = group_alloc(n);
    auto rounds = [&](int64_t C) { return ((na + C - 1) / C + ncu - 1) / ncu; };
    const int64_t c4p = 128 * (int64_t)scan4p_codes_per_slot(na);
    double best_cost = (double)rounds(c4p) * (2.30 * (double)c4p + 2065.0);
    int best = 70;
    if (n >= ((int64_t)1 << 23)) return 85;            // stretches are cut to whole rounds of the largest shape
    static const int cand[] = {85, 87, 86, 89};
    for (int v : cand) {
        const int64_t C = scan4h_codes_per_workgroup(v);
        const double cost = (double)rounds(C) * (2.45 * (double)C + 1064.0);
        if (cost < best_cost) { best_cost = cost; best = v; }
    }
    return best;
}

// M = 8 scans over regrouped codes: variants 70..79.  Variant 70 chooses the codes per lane-slot like the M = 4
// scan does: rounds * (R + 9) with rounds = ceil(workgroups / CUs) (8e6 codes: 11 rounds of 2605 workgroups at
// R = 24, 10 rounds of 2500 at R = 25, measured 12.2 ms against 11.4 ms at K = 4000).
int scan8p_codes_per_slot(int64_t n_alloc)
{
    const int ncu = cu_count();
    static const int cand[] = {25, 24, 22, 20, 18, 16};
    int best = 24;
    int64_t best_cost = INT64_MAX;
    for (int R : cand) {
        const int64_t wgs = (n_alloc + 128 * R - 1) / (128 * R);
        const int64_t cost = ((wgs + ncu - 1) / ncu) * (R + 9);
        if (cost < best_cost) { best_cost = cost; best = R; }
    }
    return best;
}

void launch_scan_grouped8(int variant, const uint4* gc8, int64_t n_alloc, const float4* img, int ntiles, int32_t* assign,
                          float* dist, hipStream_t st, RankOut ro = RankOut{}, int rpl = 0)
{
    int R = 0;
    switch (variant) {
        case 70: R = scan8p_codes_per_slot(n_alloc); break;
        case 71: launch_scan8p<12, 1024, 2>(nullptr, n_alloc, gc8, img, ntiles, assign, dist, st, ro, rpl); return;
        case 72: launch_scan8p<16, 512, 8>(nullptr, n_alloc, gc8, img, ntiles, assign, dist, st, ro, rpl); return;
        case 73: launch_scan8p<24, 512, 2>(nullptr, n_alloc, gc8, img, ntiles, assign, dist, st, ro, rpl); return;
        case 74: R = 25; break;
        case 75: R = 22; break;
        case 76: R = 20; break;
        case 77: R = 18; break;
        case 78: R = 16; break;
        default: R = 24; break;
    }
    switch (R) {
        case 16: launch_scan8p<16, 512, 4>(nullptr, n_alloc, gc8, img, ntiles, assign, dist, st, ro, rpl); break;
        case 18: launch_scan8p<18, 512, 4>(nullptr, n_alloc, gc8, img, ntiles, assign, dist, st, ro, rpl); break;
        case 20: launch_scan8p<20, 512, 4>(nullptr, n_alloc, gc8, img, ntiles, assign, dist, st, ro, rpl); break;
        case 22: launch_scan8p<22, 512, 4>(nullptr, n_alloc, gc8, img, ntiles, assign, dist, st, ro, rpl); break;
        case 25: launch_scan8p<25, 512, 4>(nullptr, n_alloc, gc8, img, ntiles, assign, dist, st, ro, rpl); break;
        default: launch_scan8p<24, 512, 4>(nullptr, n_alloc, gc8, img, ntiles, assign, dist, st, ro, rpl); break;
    }
}

// Codes per lane-slot of the two-lane M = 8 scan (a workgroup takes 256 R codes) by the rounds, in the unit of
// scan8p_codes_per_slot (128 codes' reads per tile): 2 R + 13.  24 codes per lane-slot fit the registers with the
// reads of two steps in flight instead of three (0.692 of the LDS peak against 0.686 for 22 at whole rounds; with
// three they spill and lose 8 %); 1024 threads with 10 or 8 codes per lane-slot reach 0.65 and 0.63.
int scan8q_codes_per_slot(int64_t n_alloc, int64_t* cost_out)
{
    const int ncu = cu_count();
    static const int cand[] = {24, 22, 20, 16};
    int best = 22;
    int64_t best_cost = INT64_MAX;
    for (int r : cand) {
        const int64_t wgs = (n_alloc + 256 * r - 1) / (256 * r);
        const int64_t cost = ((wgs + ncu - 1) / ncu) * (2 * r + 13);
        if (cost < best_cost) { best_cost = cost; best = r; }
    }
    if (cost_out) *cost_out = best_cost;
    return best;
}

// M = 8, many codes: four lanes per code (variant 70) or two (80), by the time the rounds take.  Per unit the
// two-lane scan is about 5 % faster (74 against 79 us at N = 1e7, K = 1e4); with few tiles its longer epilogue shows.
int choose_scan8_large(int64_t n, int K)
{
    if (K < 512) return 70;
    const int64_t na = group_alloc(n < GROUP_CHUNK_MAX - 16384 ? n : GROUP_CHUNK_MAX - 16384);
    const int ncu = cu_count();
    const int R = scan8p_codes_per_slot(na);
    const int64_t wgs = (na + 128 * R - 1) / (128 * R);
    const int64_t cost_p = ((wgs + ncu - 1) / ncu) * (R + 9);
    int64_t cost_q = 0;
    scan8q_codes_per_slot(na, &cost_q);
    return (double)cost_q * 0.95 < (double)cost_p ? 80 : 70;
}

// M = 8 scan over regrouped codes with two-lane slots (256 R codes per workgroup): variants 80..84
template <int R, int THREADS = 512, int DEPTH = 3>
void launch_scan8q_rounds(const uint4* gc8, int64_t n_alloc, const float4* img, int ntiles, int32_t* assign,
                          float* dist, hipStream_t st, RankOut ro, int rounds_per_launch)
{
    // one kernel launch per rounds_per_launch rounds of workgroups (see launch_scan4q_rounds), 0 = one for all.
    // (While the left-over groups were spread singly, a launch per round was 4 % slower for this scan: every round
    // waits for its slowest workgroup, and their conflicts made the workgroups uneven.  Placed in pairs they cost
    // half, and the two ways take the same time, 0.68 of the LDS peak at N = 1e7, K = 1e4; a launch per round moves
    // less memory.)
    constexpr int64_t C = (THREADS / 2) * (int64_t)R;
    const int64_t nwg = (n_alloc + C - 1) / C;
    const int64_t per = rounds_per_launch > 0 ? (int64_t)rounds_per_launch * cu_count() : nwg;
    for (int64_t w0 = 0; w0 < nwg; w0 += per) {
        const int64_t cnt = nwg - w0 < per ? nwg - w0 : per;
        hipLaunchKernelGGL((assign_scan8q_kernel<R, THREADS, DEPTH>), dim3((unsigned)cnt), dim3(THREADS), 0, st, n_alloc - w0 * C,
                           gc8 + w0 * C, img, ntiles, assign, dist, ro);
        ++t_scan_kernels;
    }
}

void launch_scan_grouped8_q(int variant, const uint4* gc8, int64_t n_alloc, const float4* img, int ntiles,
                            int32_t* assign, float* dist, hipStream_t st, RankOut ro, int rounds_per_launch)
{
    int R = 0;
    switch (variant) {
        case 81: R = 24; break;
        case 82: R = 22; break;
        case 83: R = 20; break;
        case 84: R = 16; break;
        default: R = scan8q_codes_per_slot(n_alloc, nullptr); break;
    }
    switch (R) {
        case 16: launch_scan8q_rounds<16>(gc8, n_alloc, img, ntiles, assign, dist, st, ro, rounds_per_launch); break;
        case 20: launch_scan8q_rounds<20>(gc8, n_alloc, img, ntiles, assign, dist, st, ro, rounds_per_launch); break;
        case 22: launch_scan8q_rounds<22>(gc8, n_alloc, img, ntiles, assign, dist, st, ro, rounds_per_launch); break;
        default: launch_scan8q_rounds<24, 512, 2>(gc8, n_alloc, img, ntiles, assign, dist, st, ro, rounds_per_launch); break;
    }
}

// the same for 64-bit codes: zero the class counters, count, plan, scatter
pqkm_status regroup_codes8(const uint8_t* codes, int64_t cnt, uint4* gc8, GroupPlan8* plan, hipStream_t st,
                           bool blocks_of_16 = false)
{
    const int64_t na = group_alloc(cnt);
    if (blocks_of_16)
        hipLaunchKernelGGL(code8_group_clear_kernel, dim3(1024), dim3(256), 0, st, gc8, na);
    hipLaunchKernelGGL(zero_u32_kernel, dim3(64), dim3(256), 0, st, plan->count, (int64_t)GROUP8_CLASSES);
    unsigned g = (unsigned)((cnt + 1023) / 1024 < 4096 ? (cnt + 1023) / 1024 : 4096);
    if (g < 1) g = 1;
    hipLaunchKernelGGL(code8_class_count_kernel, dim3(g), dim3(256), 0, st, codes, cnt, plan);
    hipLaunchKernelGGL(code8_group_plan_kernel, dim3(1), dim3(1024), 0, st, plan);
    hipLaunchKernelGGL(code8_group_scatter_kernel, dim3(g), dim3(256), 0, st, codes, cnt, plan, gc8, na,
                       blocks_of_16 ? 1 : 0);
    return launched();
}

// regroup `cnt` codes into gco: three launches on the stream
pqkm_status regroup_codes(const uint8_t* codes, int64_t cnt, uint2* gco, GroupPlan* plan, hipStream_t st,
                          bool blocks_of_16 = false)
{
    const int64_t na = group_alloc(cnt);
    if (blocks_of_16)
        hipLaunchKernelGGL(code_group_clear_kernel, dim3(1024), dim3(256), 0, st, gco, na);
    int64_t g = (cnt + 4095) / 4096;
    if (g > GROUP_MAX_WGS) g = GROUP_MAX_WGS;
    if (g < 1) g = 1;
    hipLaunchKernelGGL(code_class_count_kernel, dim3((unsigned)g), dim3(GROUP_THREADS), 0, st, codes, cnt, plan);
    hipLaunchKernelGGL(code_group_plan_kernel, dim3(1), dim3(1024), 0, st, plan, (int)g);
    hipLaunchKernelGGL(code_group_scatter_kernel, dim3((unsigned)g), dim3(GROUP_THREADS), 0, st, codes, cnt, plan, gco,
                       na, blocks_of_16 ? 1 : 0);
    return launched();
}

template <>
void launch_scan_M<4>(int variant, const uint8_t* codes, int64_t N, const float4* img, const float4* rows,
                      int ntiles, int32_t* assign, float* dist, hipStream_t st)
{
    switch (variant) {
        case 1: launch_scan<4, 16, 512, false>(codes, N, img, ntiles, assign, dist, st); break;
        case 3: launch_scan<4, 16, 512, true>(codes, N, img, ntiles, assign, dist, st); break;
        case 5: launch_scan<4, 8, 1024, false>(codes, N, img, ntiles, assign, dist, st); break;
        case 32: launch_scan4s<16, 768>(codes, N, img, ntiles, assign, dist, st); break;
        case 34: launch_scan4s<16, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        case 36: launch_scan4s<16, 512>(codes, N, img, ntiles, assign, dist, st); break;
        case 37: launch_scan4s<8, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        case 33: launch_scan4s<4, 512>(codes, N, img, ntiles, assign, dist, st); break;
        case 35: launch_scan4s<8, 512>(codes, N, img, ntiles, assign, dist, st); break;
        case 41: launch_scan4p<16, 1024, 1>(codes, N, nullptr, img, rows, ntiles, assign, dist, st); break;
        case 44: launch_scan4p<24, 512, 4>(codes, N, nullptr, img, rows, ntiles, assign, dist, st); break;
        case 46: launch_scan4p<28, 512, 3>(codes, N, nullptr, img, rows, ntiles, assign, dist, st); break;
        case 48: launch_scan4p<32, 512, 3>(codes, N, nullptr, img, rows, ntiles, assign, dist, st); break;
        default: launch_scan4s<16, 1024>(codes, N, img, ntiles, assign, dist, st); break;
    }
}
template <>
void launch_scan_M<8>(int variant, const uint8_t* codes, int64_t N, const float4* img, const float4* rows,
                      int ntiles, int32_t* assign, float* dist, hipStream_t st)
{
    switch (variant) {
        case 1: launch_scan<8, 8, 512, false>(codes, N, img, ntiles, assign, dist, st); break;
        case 2: launch_scan_skew<8, 6, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        case 3: launch_scan_skew<8, 12, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        case 4: launch_scan_skew<8, 16, 512>(codes, N, img, ntiles, assign, dist, st); break;
        case 5: launch_scan_skew<8, 24, 512>(codes, N, img, ntiles, assign, dist, st); break;
        case 6: launch_scan_skew<8, 2, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        case 7: launch_scan_skew<8, 4, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        case 40: launch_scan8p<24, 512, 4>(codes, N, nullptr, img, ntiles, assign, dist, st); break;
        case 41: launch_scan8p<12, 1024, 2>(codes, N, nullptr, img, ntiles, assign, dist, st); break;
        default: launch_scan_skew<8, 8, 1024>(codes, N, img, ntiles, assign, dist, st); break;
    }
}
template <>
void launch_scan_M<16>(int variant, const uint8_t* codes, int64_t N, const float4* img, const float4* rows,
                       int ntiles, int32_t* assign, float* dist, hipStream_t st)
{
    switch (variant) {
        case 1: launch_scan<16, 4, 512, false>(codes, N, img, ntiles, assign, dist, st); break;
        case 2: launch_scan_skew<16, 3, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        case 3: launch_scan_skew<16, 6, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        case 4: launch_scan_skew<16, 10, 512>(codes, N, img, ntiles, assign, dist, st); break;
        case 6: launch_scan_skew<16, 2, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        case 7: launch_scan_skew<16, 1, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        default: launch_scan_skew<16, 4, 1024>(codes, N, img, ntiles, assign, dist, st); break;
    }
}
template <>
void launch_scan_M<32>(int variant, const uint8_t* codes, int64_t N, const float4* img, const float4* rows,
                       int ntiles, int32_t* assign, float* dist, hipStream_t st)
{
    switch (variant) {
        case 1: launch_scan<32, 2, 512, false>(codes, N, img, ntiles, assign, dist, st); break;
        case 2: launch_scan_skew<32, 1, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        case 3: launch_scan_skew<32, 4, 1024>(codes, N, img, ntiles, assign, dist, st); break;
        case 4: launch_scan_skew<32, 6, 512>(codes, N, img, ntiles, assign, dist, st); break;
        case 5: launch_scan_skew<32, 8, 512>(codes, N, img, ntiles, assign, dist, st); break;
        case 6: launch_scan_skew<32, 1, 512>(codes, N, img, ntiles, assign, dist, st); break;
        default: launch_scan_skew<32, 2, 1024>(codes, N, img, ntiles, assign, dist, st); break;
    }
}

// Which scan runs: for M = 4 with the default variant, the regrouped half-plane scan when there is enough work
// to pay for regrouping (a pass over the codes) and the subspace-skewed scan otherwise.
inline int effective_variant(int M, int variant, int64_t N, int K, const uint8_t* codes)
{
    // the regrouped scans address the tile images through one 32-bit buffer offset: below 4 GB of images only
    const int TK = 128 / M;
    const bool img32 = (int64_t)((K + TK - 1) / TK) * TILE_BYTES < (int64_t)0xfff00000;
    const bool special = (variant >= 40 && variant <= 49) || (variant >= 70 && variant <= 79) ||
                         (M == 4 && variant >= 80 && variant <= 99) || (M == 8 && variant >= 80 && variant <= 84);
    if (M == 8) {
        const bool ok8 = img32 && ((uintptr_t)codes & 7) == 0;
        if (special && !ok8) return 0;
        // 65536 residue classes: regrouping pays once most classes hold a few dozen codes; then two lanes per code
        // (an LDS access holds two groups of four codes, so the left-over groups cost it more than the four-lane scan
        // 70, but a tile fill serves twice the codes: 0.63 against 0.60 of the LDS peak at N = 1e7, K = 1e4)
        if (variant == 0 && ok8 && K >= 256 && N >= ((int64_t)1 << 22)) return choose_scan8_large(N, K);
        if (variant == 0) {
            // skewed scan: while one round of workgroups covers the codes, the smallest shape that does so (measured
            // per round at K = 1000: 139, 172, 220, 263 us for 512, 1024, 1536, 2048 codes per workgroup)
            const int64_t ncu = cu_count();
            return N <= ncu * 512 ? 6 : N <= ncu * 1024 ? 7 : N <= ncu * 1536 ? 2 : 0;
        }
        return variant;
    }
    if ((M == 16 || M == 32) && variant == 0) {
        // the same for the wider codes (M = 16: 270, 343, 440, 524 us; M = 32: 640, 690, -, 1066 us); beyond one
        // round of those workgroups the sliding-window scan, whose workgroups take 2048 or 4096 codes
        const int64_t ncu = cu_count();
        if (M == 16) return N <= ncu * 512 ? 7 : N <= ncu * 1024 ? 6 : N <= ncu * 1536 ? 2 : 50;
        return N <= ncu * 512 ? 6 : N <= ncu * 1024 ? 2 : 50;
    }
    if (M == 4 && !img32 && special) return 34;
    if (M != 4 || variant != 0) return variant;
    // The skewed scan needs no regrouping pass and comes in shapes of 512 to 4096 codes per workgroup; a workgroup's
    // time grows with its codes (measured per round at K = 1000: 82, 107, 133, 254 us for 512, 1024, 2048, 4096),
    // so while one round of workgroups covers all codes the smallest shape that does so wins, also over the
    // regrouped scan (117 us and up per round plus the regrouping).  Beyond one round of 2048-code workgroups the
    // regrouped scan is faster; with few centers (it needs K >= 128) the two largest skewed shapes remain.
    const int64_t ncu = cu_count();
    if (N <= ncu * 512) return 33;
    if (N <= ncu * 1024) return 35;
    if (N <= ncu * 2048) return 37;
    if (K < 128 || !img32) {
        const int64_t t34 = (((N + 4095) / 4096 + ncu - 1) / ncu) * 79, t37 = (((N + 2047) / 2048 + ncu - 1) / ncu) * 42;
        return t37 < t34 ? 37 : 34;
    }
    return 70;                            // regrouped half-plane scan, codes per lane-slot chosen per launch
}
inline bool variant_grouped(int M, int variant)
{
    return ((M == 4 || M == 8) && variant >= 70 && variant <= 79) || (M == 4 && variant >= 80 && variant <= 99) ||
           (M == 8 && variant >= 80 && variant <= 84);
}
inline bool variant_two_lane(int M, int variant)
{
    return (M == 4 && variant >= 80 && variant <= 99) || (M == 8 && variant >= 80 && variant <= 84);
}
inline bool variant_table_tiles(int M, int variant) { return M == 4 && variant >= 90 && variant <= 99; }
inline bool variant_lds_loads(int M, int variant) { return M == 4 && variant >= 85 && variant <= 89; }
inline bool variant_sliding(int M, int variant) { return (M == 16 || M == 32) && variant >= 50 && variant <= 59; }

// The fused iteration's hand-over from the scan to the histogram: filled in by the caller (wanted, KT, ngroups),
// completed by the assignment (produced, nwg) when the scan that ran could file its codes by cluster group.
struct BucketLink {
    bool wanted = false, produced = false;
    int KT = 0, ngroups = 0, nwg = 0;
    // the other hand-over (sorted-path sizes): every code's rank inside its cluster, counted by the scan's epilogue
    bool rank_wanted = false, ranked = false;
};

template <int M>
pqkm_status assign_tiled(const uint8_t* codes, int64_t N, const uint8_t* centers, int K, const float* tables,
                         int32_t* assign, float* dist, float* img, const Options& opt, const Carve& c, char* ws,
                         bool reuse_groups, hipStream_t st, BucketLink* link = nullptr)
{
    constexpr int TK = 128 / M;
    int64_t ntiles = ((int64_t)K + TK - 1) / TK;
    int64_t total = ntiles * (int64_t)(TILE_BYTES / 4);
    int variant = effective_variant(M, opt.scan_variant, N, K, codes);
    // No records to file for the histogram: the four-lane scan or the scan with two-lane slots whose tiles are loaded
    // straight into LDS, half a tile ahead, in the shape that the rounds favour
    // Records to file (the fused iteration at owner-path sizes): the same scan in its 4096-code shape, which files
    // them as the four-lane scan does.
    const bool files_records = M == 4 && link && link->wanted && N <= GROUP_CHUNK_MAX - 16384 && c.bseg_off != c.pool_off;
    if (M == 4 && variant == 70 && opt.scan_variant == 0 && !files_records)
        variant = choose_scan4_large(N);
    else if (M == 4 && variant == 70 && opt.scan_variant == 0 && files_records)
        variant = 89;
    const int layout = variant_layout(M, variant);
    const bool sliding = variant_sliding(M, variant);
    if (sliding) {
        // tiles of 16 centers, plane-ordered: img[tile][m][x][16]
        ntiles = ((int64_t)K + 15) / 16;
        total = ntiles * (int64_t)16 * M * L;
        hipLaunchKernelGGL((tile_image_kernel<M, 0, 16>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           centers, K, tables, img, total);
    } else if (layout == 2 && M == 4)
        hipLaunchKernelGGL((tile_image_kernel<4, 2>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           centers, K, tables, img, total, reinterpret_cast<float*>(ws + c.rows_off));
    else if (layout == 1)
        hipLaunchKernelGGL((tile_image_kernel<M, 1>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           centers, K, tables, img, total);
    else
        hipLaunchKernelGGL((tile_image_kernel<M, 0>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           centers, K, tables, img, total);
    if (launched() != PQKM_OK) return PQKM_ERR_DEVICE;
    const bool grouped = variant_grouped(M, variant);
    int64_t per_launch = opt.launch_codes;
    // a little below the limit: with its padding a launch of exactly 2^26 codes needs one workgroup more than
    // 64 full rounds of 4096-code workgroups, and that workgroup would run a round of its own
    if ((grouped || sliding) && per_launch > GROUP_CHUNK_MAX - 16384) per_launch = GROUP_CHUNK_MAX - 16384;
    if (variant_lds_loads(M, variant)) {
        // whole rounds of these large workgroups per stretch (the regrouped copy pads a stretch by less than 32 codes)
        const int64_t round = (int64_t)cu_count() * scan4h_codes_per_workgroup(variant);
        if (per_launch >= round) per_launch = per_launch / round * round - 32;
    }
    const float4* rows = reinterpret_cast<const float4*>(ws + c.rows_off);
    uint2* gco = reinterpret_cast<uint2*>(ws + c.gco_off);
    GroupPlan* plan = reinterpret_cast<GroupPlan*>(ws + c.plan_off);
    uint4* gc8 = reinterpret_cast<uint4*>(ws + c.gc8_off);
    GroupPlan8* plan8 = reinterpret_cast<GroupPlan8*>(ws + c.plan8_off);
    // tiles built in the kernel from the transposed tables: the tables and the centers' row offsets, once per call
    TileSource tsrc{};
    if (variant_table_tiles(M, variant)) {
        float* tabT = reinterpret_cast<float*>(ws + c.tabt_off);
        uint32_t* rowoff = reinterpret_cast<uint32_t*>(ws + c.rowoff_off);
        hipLaunchKernelGGL(transpose_tables_kernel, dim3(L, (unsigned)M + 1), dim3(256), 0, st, tables, M, tabT);
        const int64_t nro = ntiles * 128;
        hipLaunchKernelGGL(tile_rows4_kernel, dim3((unsigned)((nro + 255) / 256)), dim3(256), 0, st, centers, K, rowoff, nro);
        tsrc.tabT = tabT;
        tsrc.rowoff = rowoff;
        tsrc.tab_bytes = (uint32_t)(((size_t)M * L + 1) * L * sizeof(float));
    }
    // ranks for the sorted-path histogram: from the scans that finish their codes one per lane (the regrouped scans
    // and the sliding-window scan), unless this iteration already hands records over by cluster group
    RankOut ro{};
    if (link && link->rank_wanted && (grouped || sliding) && !(M == 4 && link->wanted && variant == 70 && N <= per_launch)) {
        ro.count = reinterpret_cast<uint32_t*>(ws + c.seg_off);
        ro.rank = reinterpret_cast<uint32_t*>(ws + c.rank_off);
        unsigned zb = (unsigned)((K + 255) / 256 < 1024 ? (K + 255) / 256 : 1024);
        hipLaunchKernelGGL(zero_u32_kernel, dim3(zb), dim3(256), 0, st, ro.count, (int64_t)K);
        link->ranked = true;
    }
    for (int64_t n0 = 0; n0 < N; n0 += per_launch) {
        int64_t cnt = N - n0 < per_launch ? N - n0 : per_launch;
        const RankOut rl{ro.count, ro.count ? ro.rank + n0 : nullptr};
        // the regrouped copy survives between calls only when one launch covers all codes
        if (grouped && !(reuse_groups && N <= per_launch)) {
            const pqkm_status rs = (M == 8) ? regroup_codes8(codes + n0 * M, cnt, gc8, plan8, st, variant_two_lane(M, variant))
                                            : regroup_codes(codes + n0 * M, cnt, gco, plan, st, variant_two_lane(M, variant));
            if (rs != PQKM_OK) return PQKM_ERR_DEVICE;
        }
        EventPair ev{};
        const bool prof = (opt.profile & 1) && log_begin(g_scan_log, st, &ev);
        t_scan_kernels = 0;
        if (sliding) {
            if constexpr (M == 16 || M == 32) {
                if (launch_scan_sw<M>(variant, codes + n0 * M, cnt, reinterpret_cast<uint32_t*>(ws + c.skew_off),
                                      reinterpret_cast<const float4*>(img), (int)ntiles, assign + n0,
                                      dist ? dist + n0 : nullptr, st, rl, opt.rounds_per_launch) != PQKM_OK)
                    return PQKM_ERR_DEVICE;
            }
        } else if (M == 8 && variant_two_lane(M, variant))
            launch_scan_grouped8_q(variant, gc8, group_alloc(cnt), reinterpret_cast<const float4*>(img), (int)ntiles,
                                   assign + n0, dist ? dist + n0 : nullptr, st, rl, opt.rounds_per_launch);
        else if (variant == 89 && files_records && N <= per_launch) {
            BucketOut bo{reinterpret_cast<uint2*>(ws + c.pool_off), reinterpret_cast<uint2*>(ws + c.bseg_off), link->KT,
                         link->ngroups};
            launch_scan4h_bucket(gco, group_alloc(cnt), reinterpret_cast<const float4*>(img), rows, (int)ntiles,
                                 (K + 15) / 16, assign + n0, dist ? dist + n0 : nullptr, st, bo, &link->nwg);
            link->produced = true;
        } else if (variant_lds_loads(M, variant))
            launch_scan_grouped_h(variant, gco, group_alloc(cnt), reinterpret_cast<const float4*>(img), rows, (int)ntiles,
                                  (K + 15) / 16, assign + n0, dist ? dist + n0 : nullptr, st, rl, opt.rounds_per_launch);
        else if (variant_two_lane(M, variant))
            launch_scan_grouped_q(variant, gco, group_alloc(cnt), reinterpret_cast<const float4*>(img), rows, (int)ntiles,
                                  assign + n0, dist ? dist + n0 : nullptr, st, rl, tsrc, opt.rounds_per_launch);
        else if (grouped && M == 8)
            launch_scan_grouped8(variant, gc8, group_alloc(cnt), reinterpret_cast<const float4*>(img), (int)ntiles,
                                 assign + n0, dist ? dist + n0 : nullptr, st, rl, opt.rounds_per_launch);
        else if (grouped && M == 4 && link && link->wanted && variant == 70 && N <= per_launch &&
                 c.bseg_off != c.pool_off) {
            BucketOut bo{reinterpret_cast<uint2*>(ws + c.pool_off), reinterpret_cast<uint2*>(ws + c.bseg_off), link->KT,
                         link->ngroups};
            launch_scan_grouped(variant, gco, group_alloc(cnt), reinterpret_cast<const float4*>(img), rows,
                                (int)ntiles, assign + n0, dist ? dist + n0 : nullptr, st, &bo, &link->nwg);
            link->produced = true;
        } else if (grouped)
            launch_scan_grouped(variant, gco, group_alloc(cnt), reinterpret_cast<const float4*>(img), rows,
                                (int)ntiles, assign + n0, dist ? dist + n0 : nullptr, st, nullptr, nullptr, rl);
        else
            launch_scan_M<M>(variant, codes + n0 * M, cnt, reinterpret_cast<const float4*>(img), rows, (int)ntiles,
                             assign + n0, dist ? dist + n0 : nullptr, st);
        if (prof) {
            hipEventRecord(ev.b, st);
            std::lock_guard<std::mutex> lk(g_mu);
            g_scan_log.kernels += t_scan_kernels > 0 ? t_scan_kernels : 1;
        }
        if (launched() != PQKM_OK) return PQKM_ERR_DEVICE;
    }
    return PQKM_OK;
}

pqkm_status assign_core(const Options& opt, const Carve& c, const uint8_t* codes, int64_t N, int M,
                        const uint8_t* centers, int K, const float* tables, int32_t* assign, float* dist, void* ws,
                        hipStream_t st, bool reuse_groups, BucketLink* link)
{
    bool tiled = tiled_M(M) && opt.assign_kernel != 1 && ((uintptr_t)codes & 3) == 0;
    if (opt.assign_kernel == 2 && !tiled) return PQKM_ERR_SHAPE;
    if (!tiled) {
        hipLaunchKernelGGL(assign_generic_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, codes, N, M,
                           centers, K, tables, assign, dist);
        return launched();
    }
    float* img = reinterpret_cast<float*>(static_cast<char*>(ws) + c.img_off);
    char* wsc = static_cast<char*>(ws);
    switch (M) {
        case 4: return assign_tiled<4>(codes, N, centers, K, tables, assign, dist, img, opt, c, wsc, reuse_groups, st, link);
        case 8: return assign_tiled<8>(codes, N, centers, K, tables, assign, dist, img, opt, c, wsc, reuse_groups, st, link);
        case 16: return assign_tiled<16>(codes, N, centers, K, tables, assign, dist, img, opt, c, wsc, false, st, link);
        default: return assign_tiled<32>(codes, N, centers, K, tables, assign, dist, img, opt, c, wsc, false, st, link);
    }
}

// one whole assignment step (tile images, regrouping where it is due, scan launches), optionally bracketed by events
pqkm_status assign_impl(const Options& opt, const Carve& c, const uint8_t* codes, int64_t N, int M,
                        const uint8_t* centers, int K, const float* tables, int32_t* assign, float* dist, void* ws,
                        hipStream_t st, bool reuse_groups = false, BucketLink* link = nullptr)
{
    if (N == 0) return PQKM_OK;
    EventPair ev{};
    const bool prof = (opt.profile & 2) && log_begin(g_step_log, st, &ev);
    const pqkm_status s = assign_core(opt, c, codes, N, M, centers, K, tables, assign, dist, ws, st, reuse_groups, link);
    if (prof) hipEventRecord(ev.b, st);
    return s;
}

// counting sort of the code indices by cluster into the workspace: start[0..K] and sidx[0..#valid)
void sort_by_cluster(const int32_t* assign, int64_t N, int K, const Carve& c, char* ws, uint32_t** start_out,
                     uint32_t** sidx_out, hipStream_t st, bool ranked = false)
{
    const size_t seg_stride = align256(((size_t)K + 1) * sizeof(uint32_t));
    uint32_t* sidx = reinterpret_cast<uint32_t*>(ws + c.sidx_off);
    uint32_t* cnt = reinterpret_cast<uint32_t*>(ws + c.seg_off);
    uint32_t* start = reinterpret_cast<uint32_t*>(ws + c.seg_off + seg_stride);
    uint32_t* cursor = reinterpret_cast<uint32_t*>(ws + c.seg_off + 2 * seg_stride);
    unsigned sb = (unsigned)((N + 1023) / 1024 < 8192 ? (N + 1023) / 1024 : 8192);
    if (sb < 1) sb = 1;
    if (ranked) {
        // the scan of this iteration counted the clusters and left every code's rank: prefix, then place
        const uint32_t* rank = reinterpret_cast<const uint32_t*>(ws + c.rank_off);
        hipLaunchKernelGGL(seg_prefix_kernel, dim3(1), dim3(1024), 0, st, cnt, K, start, cursor);
        hipLaunchKernelGGL(seg_place_kernel, dim3(sb), dim3(256), 0, st, assign, rank, N, K, start, sidx);
        *start_out = start;
        *sidx_out = sidx;
        return;
    }
    unsigned zb = (unsigned)((K + 255) / 256 < 1024 ? (K + 255) / 256 : 1024);
    hipLaunchKernelGGL(zero_u32_kernel, dim3(zb), dim3(256), 0, st, cnt, (int64_t)K);
    unsigned cb = (unsigned)((N + 4095) / 4096 < 1024 ? (N + 4095) / 4096 : 1024);
    if (cb < 1) cb = 1;
    hipLaunchKernelGGL(seg_count_kernel, dim3(cb), dim3(1024), 0, st, assign, N, K, cnt);
    hipLaunchKernelGGL(seg_prefix_kernel, dim3(1), dim3(1024), 0, st, cnt, K, start, cursor);
    hipLaunchKernelGGL(seg_scatter_kernel, dim3(sb), dim3(256), 0, st, assign, N, K, start, cursor, sidx);
    *start_out = start;
    *sidx_out = sidx;
}

// does the histogram take the LDS-privatised owner path for this problem (and the call's options)?
bool owner_histogram(const HistPlan& hp, int force)
{
    return hp.KT >= 1 && hp.groups <= 255 && force != 1 && force != 3 && (force == 2 || hp.cheap);
}

// what a fused iteration asks of its assignment step: records by cluster group, when the histogram would
// otherwise take the owner path (M = 4)
BucketLink bucket_request(const Options& opt, int64_t N, int M, int K)
{
    BucketLink l;
    if (N < 1) return l;
    const HistPlan hp = hist_plan(N, M, K);
    const int force = opt.hist_kernel;
    // sorted-path sizes: the scan counts the clusters and leaves every code's rank
    if (force == 0 && !owner_histogram(hp, force) && N <= (int64_t)0xffffffff && M <= 128) l.rank_wanted = true;
    if (M != 4) return l;
    if (force != 0 || !owner_histogram(hp, force)) return l;     // a forced histogram kernel is used as named
    l.wanted = true;
    l.KT = hp.KT;
    l.ngroups = (int)hp.groups;
    return l;
}

pqkm_status update_impl(const Options& opt, const Carve& c, const uint8_t* codes, int64_t N, int M,
                        const int32_t* assign, int K, const float* tables, uint8_t* centers, uint32_t* hist,
                        uint32_t* counts, void* ws, hipStream_t st, const BucketLink* link = nullptr)
{
    if (!hist) hist = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + c.hist_off);
    if (!counts) counts = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + c.counts_off);
    const int64_t nh = (int64_t)K * M * L;
    auto zero_hist = [&]() {
        unsigned zb = (unsigned)((nh + 255) / 256 < 65536 ? (nh + 255) / 256 : 65536);
        hipLaunchKernelGGL(zero_u32_kernel, dim3(zb), dim3(256), 0, st, hist, nh);
    };
    // Owner path (LDS-privatised, no global atomics) while streaming the assignment array once per cluster
    // group is cheap; otherwise one global atomic per code and subspace into a zeroed histogram.
    const HistPlan hp = hist_plan(N, M, K);
    const int force = opt.hist_kernel;
    const bool owner = owner_histogram(hp, force);
    int S = 1;
    size_t part_stride = 0;
    uint32_t* parts = hist;
    const bool linked = owner && link && link->produced && link->KT == hp.KT && link->ngroups == (int)hp.groups;
    if (linked && M == 4 && hp.KT <= VOTE_REC_KT && link->nwg <= VOTE_REC_SEGS) {
        // the scan of this iteration filed (code, center) records by cluster group, and a vote workgroup can take
        // one group (and one subspace): it counts its histograms itself -- no histogram pass at all
        const uint2* pool = reinterpret_cast<const uint2*>(static_cast<char*>(ws) + c.pool_off);
        const uint2* bseg = reinterpret_cast<const uint2*>(static_cast<char*>(ws) + c.bseg_off);
        hipLaunchKernelGGL((vote_kernel<true>), dim3((unsigned)(hp.groups * M)), dim3(VOTE_THREADS), 0, st, hist, hist, 1,
                           (size_t)0, counts, K, M, hp.KT, tables, centers, VoteRecords{pool, bseg, link->nwg});
        return launched();
    }
    if (linked) {
        // the scan of this iteration filed (code, center) records by cluster group: count from those
        S = hp.S;
        if (S > 1) {
            parts = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + c.parts_off);
            part_stride = align256(c.hist_bytes) / sizeof(uint32_t);
        }
        const uint2* pool = reinterpret_cast<const uint2*>(static_cast<char*>(ws) + c.pool_off);
        const uint2* bseg = reinterpret_cast<const uint2*>(static_cast<char*>(ws) + c.bseg_off);
        if ((int64_t)hp.KT * M * L <= HIST_LDS_WORDS_SMALL)
            hipLaunchKernelGGL((histogram_bucket_kernel<HIST_LDS_WORDS_SMALL>), dim3((unsigned)(hp.groups * S)),
                               dim3(1024), 0, st, pool, bseg, link->nwg, K, hp.KT, S, parts, part_stride);
        else
            hipLaunchKernelGGL((histogram_bucket_kernel<HIST_LDS_WORDS>), dim3((unsigned)(hp.groups * S)), dim3(1024),
                               0, st, pool, bseg, link->nwg, K, hp.KT, S, parts, part_stride);
    } else if (owner) {
        S = hp.S;
        if (S > 1) {
            parts = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + c.parts_off);
            part_stride = align256(c.hist_bytes) / sizeof(uint32_t);
        }
        uint8_t* gid = reinterpret_cast<uint8_t*>(static_cast<char*>(ws) + c.gid_off);
        if (N > 0)
            hipLaunchKernelGGL(cluster_group_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, assign, N, K,
                               hp.KT, gid);
        if ((int64_t)hp.KT * M * L <= HIST_LDS_WORDS_SMALL)
            hipLaunchKernelGGL((histogram_owner_kernel<HIST_LDS_WORDS_SMALL>), dim3((unsigned)(hp.groups * S)),
                               dim3(1024), 0, st, codes, N, M, assign, gid, K, hp.KT, S, parts, part_stride);
        else
            hipLaunchKernelGGL((histogram_owner_kernel<HIST_LDS_WORDS>), dim3((unsigned)(hp.groups * S)), dim3(1024),
                               0, st, codes, N, M, assign, gid, K, hp.KT, S, parts, part_stride);
    } else if (force != 1 && N <= (int64_t)0xffffffff && N > 0 && M <= 128) {
        // sorted path: counting sort of the code indices by cluster, then LDS histograms per stretch of clusters
        uint32_t *start, *sidx;
        sort_by_cluster(assign, N, K, c, static_cast<char*>(ws), &start, &sidx, st, link && link->ranked);
        int KT = (HIST_LDS_WORDS / L) / M;
        if (KT > 128) KT = 128;
        hipLaunchKernelGGL(seg_hist_kernel, dim3((unsigned)((K + KT - 1) / KT)), dim3(1024), 0, st, codes, M, start, sidx,
                           K, KT, hist);
    } else {
        zero_hist();
        const int64_t per = (int64_t)1 << 30;
        for (int64_t n0 = 0; n0 < N; n0 += per) {
            int64_t cnt = N - n0 < per ? N - n0 : per;
            hipLaunchKernelGGL(histogram_atomic_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, st,
                               codes + n0 * M, cnt, M, assign + n0, K, hist);
        }
    }
    // vote: one workgroup per (subspace, CW clusters); about a thousand workgroups, at least one cluster per wave
    int64_t cw = ((int64_t)K * M + 1023) / 1024;
    cw = ((cw + 15) / 16) * 16;
    constexpr int vote_pass = VOTE_WAVES * VOTE_CPW;
    if (cw > 16) cw = ((cw + vote_pass - 1) / vote_pass) * vote_pass;   // whole passes of the waves
    if (cw > VOTE_MAX_CW) cw = VOTE_MAX_CW;
    const int64_t blocks_per_m = ((int64_t)K + cw - 1) / cw;
    hipLaunchKernelGGL((vote_kernel<false>), dim3((unsigned)(blocks_per_m * M)), dim3(VOTE_THREADS), 0, st, hist, parts, S,
                       part_stride, counts, K, M, (int)cw, tables, centers, VoteRecords{});
    return launched();
}

// workspace of the indexed assignment: sorted rows of A^0 and A^1, row minima, bucket counters / starts / cursors, items
struct IndexCarve { size_t ord_off, rowmin_off, cnt_off, start_off, cursor_off, items_off, total; };

IndexCarve index_carve(int M, int K)
{
    IndexCarve c{};
    size_t off = 0;
    c.ord_off = off;     off += align256((size_t)2 * L * L);
    c.rowmin_off = off;  off += align256((size_t)M * L * sizeof(float));
    c.cnt_off = off;     off += align256((size_t)(INDEX_BUCKETS + 1) * sizeof(uint32_t));
    c.start_off = off;   off += align256((size_t)(INDEX_BUCKETS + 1) * sizeof(uint32_t));
    c.cursor_off = off;  off += align256((size_t)(INDEX_BUCKETS + 1) * sizeof(uint32_t));
    c.items_off = off;   off += align256((size_t)K * sizeof(uint32_t));
    c.total = off;
    return c;
}

// BuildTable + FindNN of Alg. 1 with the table: files the centers, then one lane per code walks the buckets
pqkm_status assign_indexed_impl(const IndexCarve& c, const uint8_t* codes, int64_t N, int M, const uint8_t* centers, int K,
                                const float* tables, int32_t* assign, float* dist, char* ws, hipStream_t st)
{
    uint8_t* ord = reinterpret_cast<uint8_t*>(ws + c.ord_off);
    float* rowmin = reinterpret_cast<float*>(ws + c.rowmin_off);
    uint32_t* cnt = reinterpret_cast<uint32_t*>(ws + c.cnt_off);
    uint32_t* start = reinterpret_cast<uint32_t*>(ws + c.start_off);
    uint32_t* cursor = reinterpret_cast<uint32_t*>(ws + c.cursor_off);
    uint32_t* items = reinterpret_cast<uint32_t*>(ws + c.items_off);
    hipLaunchKernelGGL(index_rows_kernel, dim3(L, (unsigned)M), dim3(256), 0, st, tables, ord, rowmin);
    hipLaunchKernelGGL(zero_u32_kernel, dim3(64), dim3(256), 0, st, cnt, (int64_t)INDEX_BUCKETS);
    hipLaunchKernelGGL(index_count_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, centers, K, M, cnt);
    hipLaunchKernelGGL(seg_prefix_kernel, dim3(1), dim3(1024), 0, st, cnt, INDEX_BUCKETS, start, cursor);
    hipLaunchKernelGGL(index_scatter_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, centers, K, M, start,
                       cursor, items);
    if (N > 0)
        hipLaunchKernelGGL(assign_indexed_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, codes, N, M, centers,
                           tables, ord, rowmin, start, items, assign, dist);
    return launched();
}

template <int DS>
void launch_encode(const float* vectors, int64_t N, int M, const float* codewords, uint8_t* codes, hipStream_t st)
{
    hipLaunchKernelGGL((encode_kernel<DS, 256>), dim3((unsigned)((N + 255) / 256), (unsigned)M), dim3(256), 0, st,
                       vectors, N, M, codewords, codes);
}

}  // namespace

extern "C" {

const char* pqkm_status_string(pqkm_status s)
{
    switch (s) {
        case PQKM_OK: return "ok";
        case PQKM_ERR_NULL: return "a required pointer is NULL";
        case PQKM_ERR_SHAPE: return "invalid shape, size, alignment or option";
        case PQKM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case PQKM_ERR_DEVICE: return "not a gfx950 device, or a HIP call failed";
        case PQKM_ERR_TOO_LARGE: return "problem needs more scratch than the static buffer of pqkm_assign_noalloc holds";
    }
    return "unknown status";
}

size_t pqkm_workspace_bytes(int64_t N, int32_t M, int32_t K)
{
    if (!shape_ok(N, M, K)) return 0;
    return carve(N, M, K).total;
}

pqkm_status pqkm_build_tables(const float* codewords, int32_t M, int32_t Ds, float* tables, void* stream)
{
    if (!codewords || !tables) return PQKM_ERR_NULL;
    if (M < 1 || M > 64 || Ds < 1 || Ds > 12288) return PQKM_ERR_SHAPE;
    pqkm_status s = check_device();
    if (s != PQKM_OK) return s;
    hipLaunchKernelGGL(build_tables_kernel, dim3(L, M), dim3(256), (size_t)Ds * sizeof(float), (hipStream_t)stream,
                       codewords, Ds, tables);
    return launched();
}

pqkm_status pqkm_encode(const float* vectors, int64_t N, int32_t M, int32_t Ds, const float* codewords,
                        uint8_t* codes, void* stream)
{
    if (N < 0 || M < 1 || M > 64 || Ds < 1 || Ds > 12288 || N > (int64_t)0x7fffffff * 256) return PQKM_ERR_SHAPE;
    if (!codewords || (N > 0 && (!vectors || !codes))) return PQKM_ERR_NULL;
    pqkm_status s = check_device();
    if (s != PQKM_OK) return s;
    if (N == 0) return PQKM_OK;
    hipStream_t st = (hipStream_t)stream;
    switch (Ds) {
        case 4: launch_encode<4>(vectors, N, M, codewords, codes, st); break;
        case 8: launch_encode<8>(vectors, N, M, codewords, codes, st); break;
        case 16: launch_encode<16>(vectors, N, M, codewords, codes, st); break;
        case 32: launch_encode<32>(vectors, N, M, codewords, codes, st); break;
        case 64: launch_encode<64>(vectors, N, M, codewords, codes, st); break;
        case 128: launch_encode<128>(vectors, N, M, codewords, codes, st); break;
        default:
            hipLaunchKernelGGL(encode_generic_kernel, dim3((unsigned)((N + 255) / 256), (unsigned)M), dim3(256), 0, st,
                               vectors, N, M, Ds, codewords, codes);
    }
    return launched();
}

pqkm_status pqkm_decode(const uint8_t* codes, int64_t N, int32_t M, int32_t Ds, const float* codewords,
                        float* vectors, void* stream)
{
    if (N < 0 || M < 1 || M > 64 || Ds < 1 || Ds > 12288) return PQKM_ERR_SHAPE;
    if (!codewords || (N > 0 && (!vectors || !codes))) return PQKM_ERR_NULL;
    pqkm_status s = check_device();
    if (s != PQKM_OK) return s;
    if (N == 0) return PQKM_OK;
    const int64_t total = N * M * Ds;
    if ((total + 255) / 256 > (int64_t)0x7fffffff) return PQKM_ERR_SHAPE;
    hipLaunchKernelGGL(decode_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream, codes,
                       total, M, Ds, codewords, vectors);
    return launched();
}

pqkm_status pqkm_assign(const uint8_t* codes, int64_t N, int32_t M, const uint8_t* centers, int32_t K,
                        const float* tables, int32_t* assign, float* dist, void* workspace, size_t workspace_bytes,
                        void* stream)
{
    if (!shape_ok(N, M, K)) return PQKM_ERR_SHAPE;
    if (!centers || !tables || (N > 0 && (!codes || !assign))) return PQKM_ERR_NULL;
    const Carve c = carve(N, M, K);
    pqkm_status s = check_workspace(workspace, workspace_bytes, c.total);
    if (s != PQKM_OK) return s;
    if ((s = check_device()) != PQKM_OK) return s;
    return assign_impl(options_snapshot(), c, codes, N, M, centers, K, tables, assign, dist, workspace,
                       (hipStream_t)stream);
}

pqkm_status pqkm_assign_noalloc(const uint8_t* codes, int64_t N, int32_t M, const uint8_t* centers, int32_t K,
                                const float* tables, int32_t* assign, float* dist, void* stream)
{
    if (!shape_ok(N, M, K)) return PQKM_ERR_SHAPE;
    if (!centers || !tables || (N > 0 && (!codes || !assign))) return PQKM_ERR_NULL;
    const Carve c = carve(N, M, K);
    if (c.total > (size_t)PQKM_NOALLOC_SCRATCH_BYTES) return PQKM_ERR_TOO_LARGE;
    pqkm_status s = check_device();
    if (s != PQKM_OK) return s;
    void* ws = nullptr;
    if ((s = scratch_of_current_device(&ws)) != PQKM_OK) return s;
    Options opt = options_snapshot();
    opt.profile = 0;                        // the event pairs of the profile option are created on demand
    return assign_impl(opt, c, codes, N, M, centers, K, tables, assign, dist, ws, (hipStream_t)stream);
}

size_t pqkm_index_workspace_bytes(int32_t M, int32_t K)
{
    if (M < 2 || M > 64 || K < 1) return 0;
    return index_carve(M, K).total;
}

pqkm_status pqkm_assign_indexed(const uint8_t* codes, int64_t N, int32_t M, const uint8_t* centers, int32_t K,
                                const float* tables, int32_t* assign, float* dist, void* workspace,
                                size_t workspace_bytes, void* stream)
{
    if (!shape_ok(N, M, K) || M < 2 || N > (int64_t)0x7fffffff * 256) return PQKM_ERR_SHAPE;
    if (!centers || !tables || (N > 0 && (!codes || !assign))) return PQKM_ERR_NULL;
    const IndexCarve c = index_carve(M, K);
    pqkm_status s = check_workspace(workspace, workspace_bytes, c.total);
    if (s != PQKM_OK) return s;
    if ((s = check_device()) != PQKM_OK) return s;
    return assign_indexed_impl(c, codes, N, M, centers, K, tables, assign, dist, static_cast<char*>(workspace),
                               (hipStream_t)stream);
}

size_t pqkm_check_workspace_bytes(int64_t n_sample, int32_t M, int32_t K)
{
    if (!shape_ok(n_sample, M, K) || M < 2) return 0;
    const size_t a = carve(n_sample, M, K).total, b = index_carve(M, K).total;
    return (a > b ? a : b) + align256((size_t)n_sample * sizeof(int32_t));
}

pqkm_status pqkm_check(const uint8_t* sample_codes, int64_t n_sample, int32_t M, const uint8_t* centers, int32_t K,
                       const float* tables, int32_t trials, void* workspace, size_t workspace_bytes, void* stream,
                       int32_t* use_index, float* scan_ms, float* index_ms)
{
    if (!shape_ok(n_sample, M, K) || M < 2 || n_sample < 1 || trials < 1) return PQKM_ERR_SHAPE;
    if (!centers || !tables || !sample_codes || !use_index) return PQKM_ERR_NULL;
    const Carve ca = carve(n_sample, M, K);
    const IndexCarve ci = index_carve(M, K);
    const size_t shared = ca.total > ci.total ? ca.total : ci.total;
    pqkm_status s = check_workspace(workspace, workspace_bytes, shared + align256((size_t)n_sample * sizeof(int32_t)));
    if (s != PQKM_OK) return s;
    if ((s = check_device()) != PQKM_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    char* ws = static_cast<char*>(workspace);
    int32_t* out = reinterpret_cast<int32_t*>(ws + shared);
    Options opt = options_snapshot();
    opt.profile = 0;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return PQKM_ERR_DEVICE;
    if (hipEventCreate(&e1) != hipSuccess) { hipEventDestroy(e0); return PQKM_ERR_DEVICE; }
    float best_ms[2] = {0.f, 0.f};
    for (int which = 0; which < 2 && s == PQKM_OK; ++which) {
        for (int t = 0; t <= trials && s == PQKM_OK; ++t) {          // trial 0 is a warm-up and is not counted
            if (hipEventRecord(e0, st) != hipSuccess) { s = PQKM_ERR_DEVICE; break; }
            s = which == 0 ? assign_impl(opt, ca, sample_codes, n_sample, M, centers, K, tables, out, nullptr, ws, st)
                           : assign_indexed_impl(ci, sample_codes, n_sample, M, centers, K, tables, out, nullptr, ws, st);
            if (s != PQKM_OK) break;
            float ms = 0.f;
            if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { s = PQKM_ERR_DEVICE; break; }
            if (t == 1 || (t > 1 && ms < best_ms[which])) best_ms[which] = ms;
        }
    }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (s != PQKM_OK) return s;
    if (scan_ms) *scan_ms = best_ms[0];
    if (index_ms) *index_ms = best_ms[1];
    *use_index = best_ms[1] < best_ms[0] ? 1 : 0;
    return PQKM_OK;
}

pqkm_status pqkm_update(const uint8_t* codes, int64_t N, int32_t M, const int32_t* assign, int32_t K,
                        const float* tables, uint8_t* centers, uint32_t* hist, uint32_t* counts, void* workspace,
                        size_t workspace_bytes, void* stream)
{
    if (!shape_ok(N, M, K)) return PQKM_ERR_SHAPE;
    if (!centers || !tables || (N > 0 && (!codes || !assign))) return PQKM_ERR_NULL;
    const Carve c = carve(N, M, K);
    pqkm_status s = check_workspace(workspace, workspace_bytes, c.total);
    if (s != PQKM_OK) return s;
    if ((s = check_device()) != PQKM_OK) return s;
    return update_impl(options_snapshot(), c, codes, N, M, assign, K, tables, centers, hist, counts, workspace,
                       (hipStream_t)stream);
}

pqkm_status pqkm_update_naive(const uint8_t* codes, int64_t N, int32_t M, const int32_t* assign, int32_t K,
                              const float* tables, uint8_t* centers, double* cost, void* workspace,
                              size_t workspace_bytes, void* stream)
{
    if (!shape_ok(N, M, K) || N > (int64_t)0xffffffff) return PQKM_ERR_SHAPE;
    if (!centers || !tables || (N > 0 && (!codes || !assign))) return PQKM_ERR_NULL;
    const Carve c = carve(N, M, K);
    pqkm_status s = check_workspace(workspace, workspace_bytes, c.total);
    if (s != PQKM_OK) return s;
    if ((s = check_device()) != PQKM_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    uint32_t *start, *sidx;
    sort_by_cluster(assign, N, K, c, static_cast<char*>(workspace), &start, &sidx, st);
    // grid (K, M): K up to 2^31 - 1 fits the x dimension
    hipLaunchKernelGGL(naive_update_kernel, dim3((unsigned)K, (unsigned)M), dim3(256), 0, st, codes, M, start, sidx,
                       tables, centers, cost);
    return launched();
}

pqkm_status pqkm_fit(const uint8_t* codes, int64_t N, int32_t M, const float* tables, int32_t K, uint8_t* centers,
                     int32_t iters, int32_t* assign, uint32_t* hist, uint32_t* counts, void* workspace,
                     size_t workspace_bytes, void* stream)
{
    if (!shape_ok(N, M, K) || iters < 0) return PQKM_ERR_SHAPE;
    if (!centers || !tables || (N > 0 && (!codes || !assign))) return PQKM_ERR_NULL;
    const Carve c = carve(N, M, K);
    pqkm_status s = check_workspace(workspace, workspace_bytes, c.total);
    if (s != PQKM_OK) return s;
    if ((s = check_device()) != PQKM_OK) return s;
    const Options opt = options_snapshot();
    for (int it = 0; it < iters; ++it) {
        // the codes do not change between iterations: regroup them for the scan once
        BucketLink link = bucket_request(opt, N, M, K);
        s = assign_impl(opt, c, codes, N, M, centers, K, tables, assign, nullptr, workspace, (hipStream_t)stream, it > 0,
                        &link);
        if (s != PQKM_OK) return s;
        s = update_impl(opt, c, codes, N, M, assign, K, tables, centers, hist, counts, workspace, (hipStream_t)stream,
                        &link);
        if (s != PQKM_OK) return s;
    }
    return PQKM_OK;
}

// extra workspace of pqkm_fit_until, placed after the pqkm_fit carve
struct UntilCarve { size_t prev_off, dist_off, pa_off, ph_off, out_off, total; };

static UntilCarve until_carve(int64_t N, int M, int K)
{
    UntilCarve u{};
    size_t off = carve(N, M, K).total;
    u.prev_off = off;  off += align256((size_t)N * sizeof(int32_t));
    u.dist_off = off;  off += align256((size_t)N * sizeof(float));
    u.pa_off = off;    off += align256((size_t)STAT_BLOCKS * sizeof(StatPartial));
    u.ph_off = off;    off += align256((size_t)STAT_BLOCKS * sizeof(StatPartial));
    u.out_off = off;   off += 256;
    u.total = off;
    return u;
}

size_t pqkm_fit_until_workspace_bytes(int64_t N, int32_t M, int32_t K)
{
    if (!shape_ok(N, M, K)) return 0;
    return until_carve(N, M, K).total;
}

pqkm_status pqkm_fit_until(const uint8_t* codes, int64_t N, int32_t M, const float* tables, int32_t K,
                           uint8_t* centers, int32_t max_iters, int32_t* assign, uint32_t* hist, uint32_t* counts,
                           pqkm_iter_stats* stats, int32_t* iters_done, void* workspace, size_t workspace_bytes,
                           void* stream)
{
    if (!shape_ok(N, M, K) || max_iters < 0) return PQKM_ERR_SHAPE;
    if (!centers || !tables || (N > 0 && (!codes || !assign))) return PQKM_ERR_NULL;
    const UntilCarve u = until_carve(N, M, K);
    pqkm_status s = check_workspace(workspace, workspace_bytes, u.total);
    if (s != PQKM_OK) return s;
    if ((s = check_device()) != PQKM_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    char* ws = static_cast<char*>(workspace);
    const Carve c = carve(N, M, K);
    int32_t* prev = reinterpret_cast<int32_t*>(ws + u.prev_off);
    float* dist = reinterpret_cast<float*>(ws + u.dist_off);
    StatPartial* pa = reinterpret_cast<StatPartial*>(ws + u.pa_off);
    StatPartial* ph = reinterpret_cast<StatPartial*>(ws + u.ph_off);
    unsigned long long* out = reinterpret_cast<unsigned long long*>(ws + u.out_off);
    if (!hist) hist = reinterpret_cast<uint32_t*>(ws + c.hist_off);
    if (!counts) counts = reinterpret_cast<uint32_t*>(ws + c.counts_off);
    if (iters_done) *iters_done = 0;
    if (N > 0) {
        unsigned fb = (unsigned)((N + 255) / 256 < 65536 ? (N + 255) / 256 : 65536);
        hipLaunchKernelGGL(fill_i32_kernel, dim3(fb), dim3(256), 0, st, prev, N, (int32_t)-1);
    }
    const Options opt = options_snapshot();
    for (int it = 0; it < max_iters; ++it) {
        BucketLink link = bucket_request(opt, N, M, K);
        s = assign_impl(opt, c, codes, N, M, centers, K, tables, assign, dist, workspace, st, it > 0, &link);
        if (s != PQKM_OK) return s;
        hipLaunchKernelGGL(iter_assign_stats_kernel, dim3(STAT_BLOCKS), dim3(256), 0, st, assign, prev, dist, N, pa);
        s = update_impl(opt, c, codes, N, M, assign, K, tables, centers, hist, counts, workspace, st, &link);
        if (s != PQKM_OK) return s;
        hipLaunchKernelGGL(iter_hist_stats_kernel, dim3(STAT_BLOCKS), dim3(256), 0, st, hist, (int64_t)K * M * L,
                           counts, K, ph);
        hipLaunchKernelGGL(iter_stats_final_kernel, dim3(1), dim3(64), 0, st, pa, ph, out);
        unsigned long long h[4];
        if (hipMemcpyAsync(h, out, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess) return PQKM_ERR_DEVICE;
        if (hipStreamSynchronize(st) != hipSuccess) return PQKM_ERR_DEVICE;
        if (stats) {
            double d;
            memcpy(&d, &h[0], sizeof(d));
            stats[it].objective = d;
            stats[it].changed = (int64_t)h[1];
            stats[it].nonzero_bins = (int64_t)h[2];
            stats[it].nonempty = (int64_t)h[3];
        }
        if (iters_done) *iters_done = it + 1;
        if (h[1] == 0) break;
    }
    return PQKM_OK;
}

pqkm_status pqkm_set_option(const char* name, int32_t value)
{
    if (!name) return PQKM_ERR_NULL;
    std::lock_guard<std::mutex> lk(g_mu);
    if (strcmp(name, "assign_kernel") == 0) {
        if (value < 0 || value > 2) return PQKM_ERR_SHAPE;
        g_opt.assign_kernel = value;
    } else if (strcmp(name, "scan_variant") == 0) {
        if (value < 0 || value > 99) return PQKM_ERR_SHAPE;
        g_opt.scan_variant = value;
    } else if (strcmp(name, "hist_kernel") == 0) {
        if (value < 0 || value > 3) return PQKM_ERR_SHAPE;
        g_opt.hist_kernel = value;
    } else if (strcmp(name, "profile") == 0) {
        if (value < 0 || value > 3) return PQKM_ERR_SHAPE;
        g_opt.profile = value;
    } else if (strcmp(name, "scan_rounds_per_launch") == 0) {
        if (value < 0 || value > 1024) return PQKM_ERR_SHAPE;
        g_opt.rounds_per_launch = value;
    } else if (strcmp(name, "launch_codes_log2") == 0) {
        if (value < 10 || value > 40) return PQKM_ERR_SHAPE;
        g_opt.launch_codes = (int64_t)1 << value;
    } else {
        return PQKM_ERR_SHAPE;
    }
    return PQKM_OK;
}

pqkm_status pqkm_profile_read(double* total_ms, int64_t* launches)
{
    return log_read(g_scan_log, total_ms, launches);
}

pqkm_status pqkm_profile_read_steps(double* total_ms, int64_t* steps)
{
    return log_read(g_step_log, total_ms, steps);
}

}  // extern "C"
