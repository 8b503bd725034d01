// HIP kernels for the PQk-means iteration on gfx950 (wave64, 160 KB LDS per CU).
//
// Naming follows the paper: A^m are the per-subspace 256x256 distance tables
// (Sec. 2.2), SDC is the squared symmetric distance (Eq. 3), the assignment is
// Eq. 5, the histogram Eq. 7 and the vote Eq. 8.
//
// Everything here is compiled with -ffp-contract=off: the only fused operation
// is the explicit fmaf of the vote.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pqkm {

constexpr int L = 256;                    // subcodewords per subspace
constexpr int TILE_BYTES = 128 * 1024;    // LDS image of one center tile
constexpr int TILE_F4 = TILE_BYTES / 16;  // the same in float4 units
constexpr int IDX_NONE = 0x7fffffff;      // "no center improved yet"

// ---------------------------------------------------------------------------------------------
// Sec. 2.2: A^m[i][j] = || c^m_i - c^m_j ||^2, fp64 accumulation in ascending dimension, direct
// difference form, one rounding to fp32.  Grid (256, M), block 256: block (i, m), thread j.
// Codeword i is staged in LDS; codeword j is read with stride Ds (small, cache resident).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void build_tables_kernel(const float* __restrict__ codewords, int Ds,
                                                           float* __restrict__ tables)
{
    extern __shared__ float ci[];
    const int i = blockIdx.x, m = blockIdx.y, j = threadIdx.x;
    const float* cw = codewords + (size_t)m * L * Ds;
    for (int d = j; d < Ds; d += 256) ci[d] = cw[(size_t)i * Ds + d];
    __syncthreads();
    const float* cj = cw + (size_t)j * Ds;
    double acc = 0.0;
    for (int d = 0; d < Ds; ++d) {
        double diff = (double)ci[d] - (double)cj[d];
        double sq = diff * diff;
        acc = acc + sq;
    }
    tables[((size_t)m * L + i) * L + j] = (float)acc;
}

// ---------------------------------------------------------------------------------------------
// Sec. 2.2, encoding: every subvector is replaced by the index of its closest codeword.  Distance:
// fp32, ascending dimension, one subtraction and one fused multiply-add per dimension (explicit
// fmaf; the file is compiled without contraction); ties go to the lowest index (strict "<" over
// ascending l).  Grid (blocks of THREADS vectors, M), one thread per vector: the subvector sits in
// registers; the codewords are the same for every lane, so the scalar unit fetches them (s_load
// through the constant cache) and each subtraction takes one as its scalar source: no LDS, no
// vector loads in the loop; four codewords in flight for instruction-level parallelism.  Plain
// VALU work, 3 flops per (vector, codeword, dimension); an MFMA formulation through
// ||x||^2 - 2 x.c + ||c||^2 would round differently and could not be compared bit for bit.
// ---------------------------------------------------------------------------------------------
template <int DS, int THREADS>
__global__ __launch_bounds__(THREADS) void encode_kernel(const float* __restrict__ vectors, int64_t N, int M,
                                                           const float* __restrict__ codewords,
                                                           uint8_t* __restrict__ codes)
{
    const int m = blockIdx.y;
    const float* __restrict__ cw = codewords + (size_t)m * L * DS;      // uniform
    int64_t n = (int64_t)blockIdx.x * THREADS + threadIdx.x;
    const bool live = n < N;
    if (!live) n = N - 1;
    float x[DS];
    const float* xv = vectors + ((size_t)n * M + m) * DS;
#pragma unroll
    for (int d = 0; d < DS; ++d) x[d] = xv[d];
    float best = INFINITY;
    int bl = 0;
    for (int l0 = 0; l0 < L; l0 += 4) {
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int d = 0; d < DS; ++d) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float t = x[d] - cw[(l0 + u) * DS + d];
                acc[u] = __builtin_fmaf(t, t, acc[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (acc[u] < best) {
                best = acc[u];
                bl = l0 + u;
            }
    }
    if (live) codes[n * M + m] = (uint8_t)bl;
}

// any subvector length: same arithmetic, operands read through the caches
__global__ __launch_bounds__(256) void encode_generic_kernel(const float* __restrict__ vectors, int64_t N, int M,
                                                             int Ds, const float* __restrict__ codewords,
                                                             uint8_t* __restrict__ codes)
{
    const int m = blockIdx.y;
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    const float* xv = vectors + ((size_t)n * M + m) * Ds;
    float best = INFINITY;
    int bl = 0;
    for (int l = 0; l < L; ++l) {
        const float* c = codewords + ((size_t)m * L + l) * Ds;
        float acc = 0.0f;
        for (int d = 0; d < Ds; ++d) {
            const float t = xv[d] - c[d];
            acc = __builtin_fmaf(t, t, acc);
        }
        if (acc < best) {
            best = acc;
            bl = l;
        }
    }
    codes[n * M + m] = (uint8_t)bl;
}

// Sec. 2.2, reconstruction: a code decodes to the concatenation of its codewords.  One thread per output element.
__global__ __launch_bounds__(256) void decode_kernel(const uint8_t* __restrict__ codes, int64_t total, int M, int Ds,
                                                     const float* __restrict__ codewords, float* __restrict__ out)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int d = (int)(e % Ds);
    const int64_t nm = e / Ds;
    const int m = (int)(nm % M);
    out[e] = codewords[((size_t)m * L + codes[nm]) * Ds + d];
}

// ---------------------------------------------------------------------------------------------
// Generic assignment (any M): one lane per code, centers read wave-uniformly, table entries
// gathered through the cache hierarchy.  Eq. 5 exactly as written: ascending k, strict <.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void assign_generic_kernel(const uint8_t* __restrict__ codes, int64_t N, int M,
                                                             const uint8_t* __restrict__ centers, int K,
                                                             const float* __restrict__ tables,
                                                             int32_t* __restrict__ assign, float* __restrict__ dist)
{
    int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    const uint8_t* x = codes + n * M;
    float best = INFINITY;
    int bk = 0;
    for (int k = 0; k < K; ++k) {
        const uint8_t* mu = centers + (size_t)k * M;
        float s = tables[((size_t)0 * L + x[0]) * L + mu[0]];
        for (int m = 1; m < M; ++m) {
            float a = tables[((size_t)m * L + x[m]) * L + mu[m]];
            s = s + a;
        }
        if (s < best) {
            best = s;
            bk = k;
        }
    }
    assign[n] = bk;
    if (dist) dist[n] = best;
}

// ---------------------------------------------------------------------------------------------
// Center-tile images for the LDS-tiled scan.
//
// A tile holds TK = 128 / M consecutive centers.  Its image is laid out exactly as the scan
// wants it in LDS:   img[tile][m][x][kin] = A^m[x][centers[tile*TK + kin][m]]      (fp32)
// i.e. for every subspace m and possible code subcode x, one contiguous row of TK entries (one
// per center of the tile).  A row is TK*4 bytes, a tile 128 KB.  With x in the low address
// bits, the rows two codes read in the same subspace fall on LDS banks chosen by their
// subcodes rather than all on the same ones.  Centers past K are padded with +inf, which a
// strict "<" never selects.  One thread per element, kin fastest, so stores are contiguous.
// ---------------------------------------------------------------------------------------------
// LAYOUT 1 is the alternative order img[tile][x][m][kin] used by the subspace-skewed scan, in which
// the LDS bank half of a row is decided by the parity of m instead of the parity of x.  LAYOUT 2
// (M = 4, TK = 32 only) is img[tile][m][h][x][kin % 16] with h = kin / 16: eight planes of 16 KB.
// With LAYOUT 2 the kernel can also write a second copy of the images in the order of LAYOUT 0.
template <int M, int LAYOUT = 0, int TK = 128 / M>
__global__ __launch_bounds__(256) void tile_image_kernel(const uint8_t* __restrict__ centers, int K,
                                                         const float* __restrict__ tables, float* __restrict__ img,
                                                         int64_t total, float* __restrict__ rows = nullptr)
{
    int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    int kin = (int)(e % TK);
    int x, m;
    if (LAYOUT == 2) {
        const int h = (int)((e / (16 * L)) % 2);
        kin = (int)(e % 16) + 16 * h;
        x = (int)((e / 16) % L);
        m = (int)((e / (32 * L)) % M);
    } else if (LAYOUT == 1) {
        m = (int)((e / TK) % M);
        x = (int)((e / (TK * M)) % L);
    } else {
        x = (int)((e / TK) % L);
        m = (int)((e / (TK * L)) % M);
    }
    int64_t tile = e / ((int64_t)TK * M * L);
    int64_t k = tile * TK + kin;
    float v = INFINITY;
    if (k < K) v = tables[((size_t)m * L + x) * L + centers[k * M + m]];
    img[e] = v;
    // second copy in the plain order [tile][m][x][k] (LAYOUT 2 only): one 128-byte line per (tile, m, x), read by
    // the epilogue of the half-plane scan
    if (LAYOUT == 2 && rows) rows[((tile * M + m) * L + x) * TK + kin] = v;
}

// ---------------------------------------------------------------------------------------------
// LDS-tiled assignment scan (Eq. 5 over Eq. 3), M in {4, 8, 16, 32}.
//
// Work decomposition.  A workgroup keeps C = SLOTS*R codes in registers and walks over all
// center tiles; each tile image is copied from global memory into LDS once per workgroup and
// then serves C * TK distance evaluations.  LPS = TK/4 consecutive lanes form a "slot" that
// works on one code at a time: lane q of the slot reads, for every subspace m, the 16 bytes
//      tile[m][x_m][4q .. 4q+3]          (one ds_read_b128)
// so the LPS lanes of a slot read one contiguous row and different slots read different rows:
// the M gathers per (code, center) of Eq. 3 become M/4 wide LDS reads per lane with no address
// arithmetic in the loop (the per-code byte offsets of the M rows are computed once and kept
// in registers when M = 4; for larger M they are rebuilt from the packed code).
//
// Each lane sums its 4 centers in ascending m (fp32, unfused) and keeps the running minimum and
// its index over the centers it sees; since it sees them in ascending k, a strict "<" keeps the
// lowest index.  At the end the LPS lanes of a slot are merged by (value, index) with xor
// shuffles -- the wavefront-level argmin -- and lane 0 of the slot writes the result.
// ---------------------------------------------------------------------------------------------
template <int M> struct ScanShape {
    static constexpr int TK = 128 / M;      // centers per tile
    static constexpr int LPS = TK / 4;      // lanes per slot
    static constexpr int ROWB = TK * 4;     // bytes per (m, x) row
    static constexpr int MB = L * ROWB;     // bytes per subspace
    static constexpr int W = M / 4;         // 32-bit words per packed code
};

__device__ __forceinline__ float4 lds_read16(const char* base, uint32_t byte_off)
{
    return *reinterpret_cast<const float4*>(base + byte_off);
}

template <int M, int R, int THREADS, bool PREFETCH>
__global__ __launch_bounds__(THREADS) void assign_scan_kernel(const uint8_t* __restrict__ codes, int64_t N,
                                                              const float4* __restrict__ img, int ntiles,
                                                              int32_t* __restrict__ assign,
                                                              float* __restrict__ dist)
{
    using S = ScanShape<M>;
    constexpr int SLOTS = THREADS / S::LPS;
    constexpr int C = SLOTS * R;
    constexpr int NF = TILE_F4 / THREADS;   // float4 per thread per tile fill
    static_assert(TILE_F4 % THREADS == 0, "tile must divide evenly over the workgroup");

    __shared__ float4 tile[TILE_F4];
    const char* tb = reinterpret_cast<const char*>(tile);

    const int tid = threadIdx.x;
    const int q = tid % S::LPS;
    const int c = tid / S::LPS;
    const int64_t base = (int64_t)blockIdx.x * C;

    uint32_t pk[R][S::W];
    float best[R];
    int idx[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t n = base + (int64_t)r * SLOTS + c;
        if (n >= N) n = N - 1;
        const uint32_t* cw = reinterpret_cast<const uint32_t*>(codes + n * M);
#pragma unroll
        for (int w = 0; w < S::W; ++w) pk[r][w] = cw[w];
        best[r] = INFINITY;
        idx[r] = IDX_NONE;
    }
    // M = 4: per-code LDS byte offsets, fixed for the whole kernel
    uint32_t off[R][4];
    if (M == 4) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int m = 0; m < 4; ++m) off[r][m] = m * S::MB + ((pk[r][0] >> (8 * m)) & 255u) * S::ROWB + q * 16;
    }

    float4 pf[NF];
    if (PREFETCH) {
#pragma unroll
        for (int i = 0; i < NF; ++i) pf[i] = img[(size_t)i * THREADS + tid];
    }

    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();                       // everyone is done reading the previous tile
        if (PREFETCH) {
#pragma unroll
            for (int i = 0; i < NF; ++i) tile[i * THREADS + tid] = pf[i];
        } else {
            const float4* src = img + (size_t)t * TILE_F4;
#pragma unroll
            for (int i = 0; i < NF; ++i) tile[i * THREADS + tid] = src[(size_t)i * THREADS + tid];
        }
        __syncthreads();
        if (PREFETCH && t + 1 < ntiles) {
            const float4* src = img + (size_t)(t + 1) * TILE_F4;
#pragma unroll
            for (int i = 0; i < NF; ++i) pf[i] = src[(size_t)i * THREADS + tid];
        }
        const int kb = t * S::TK + q * 4;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float4 s;
            if (M == 4) {
                float4 v0 = lds_read16(tb, off[r][0]);
                float4 v1 = lds_read16(tb, off[r][1]);
                float4 v2 = lds_read16(tb, off[r][2]);
                float4 v3 = lds_read16(tb, off[r][3]);
                s.x = v0.x + v1.x; s.y = v0.y + v1.y; s.z = v0.z + v1.z; s.w = v0.w + v1.w;
                s.x = s.x + v2.x;  s.y = s.y + v2.y;  s.z = s.z + v2.z;  s.w = s.w + v2.w;
                s.x = s.x + v3.x;  s.y = s.y + v3.y;  s.z = s.z + v3.z;  s.w = s.w + v3.w;
            } else {
#pragma unroll
                for (int m = 0; m < M; ++m) {
                    uint32_t x = (pk[r][m / 4] >> (8 * (m % 4))) & 255u;
                    float4 v = lds_read16(tb, x * S::ROWB + q * 16 + m * S::MB);
                    if (m == 0) {
                        s = v;
                    } else {
                        s.x = s.x + v.x; s.y = s.y + v.y; s.z = s.z + v.z; s.w = s.w + v.w;
                    }
                }
            }
            float b = best[r];
            int bi = idx[r];
            if (s.x < b) { b = s.x; bi = kb; }
            if (s.y < b) { b = s.y; bi = kb + 1; }
            if (s.z < b) { b = s.z; bi = kb + 2; }
            if (s.w < b) { b = s.w; bi = kb + 3; }
            best[r] = b;
            idx[r] = bi;
        }
    }

    // wavefront-level argmin over the lanes of a slot: smaller value, then smaller index
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float b = best[r];
        int bi = idx[r];
#pragma unroll
        for (int d = S::LPS / 2; d >= 1; d >>= 1) {
            float ob = __shfl_xor(b, d);
            int oi = __shfl_xor(bi, d);
            if (ob < b || (ob == b && oi < bi)) { b = ob; bi = oi; }
        }
        int64_t n = base + (int64_t)r * SLOTS + c;
        if (q == 0 && n < N) {
            assign[n] = (bi == IDX_NONE) ? 0 : bi;
            if (dist) dist[n] = b;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Helpers of the M = 4 scans (32-bit SIFT-like codes are the paper's main workload, Tab. 3 and
// Tab. 5).  These kernels are tuned for the register file:
//
//  * per code and lane only a few registers persist: words of packed, pre-scaled LDS row offsets
//    (16-bit fields, byte offset / 16; one SDWA shift unpacks a field), the running minimum and
//    the index of the TILE in which it last improved;
//  * the minimum over the lane's centers of a tile is tracked with v_min3 and one compare; which
//    center of that tile attains it is recovered once, after the last tile, by re-reading the
//    terms of those sums from the tile image in global memory (same bits, same sum order) and
//    taking the first equal one -- the same center a sequential strict "<" scan would keep;
//  * LDS reads run ahead of the sums that consume them;
//  * the next tile is prefetched from global memory into registers while the current one is
//    being scanned, so only the LDS write of the fill is exposed between two barriers.
// ---------------------------------------------------------------------------------------------
// Field unpacks that issue at the full VALU rate.  Measured on this chip: v_and_b32, v_lshrrev_b32, v_add_u32
// and the fp32 add / mul / fma issue every 2.4 clocks per SIMD; v_lshlrev_b32 (also as SDWA), v_min/max/min3,
// v_bfe_u32 and the other three-operand integer forms every 4.2.  A register holds a 15-bit byte offset in its low
// bits and a 17-bit byte offset from bit 15 up.
__device__ __forceinline__ uint32_t unpack_low15(uint32_t mask7fff, uint32_t v)
{
    uint32_t r;
    asm volatile("v_and_b32 %0, %1, %2" : "=v"(r) : "s"(mask7fff), "v"(v));
    return r;
}
__device__ __forceinline__ uint32_t unpack_high17(uint32_t v)
{
    uint32_t r;
    asm volatile("v_lshrrev_b32 %0, 15, %1" : "=v"(r) : "v"(v));
    return r;
}
__device__ __forceinline__ uint32_t sdwa_shl_word0(uint32_t sh, uint32_t v)
{
    uint32_t r;
    asm volatile("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0"
        : "=v"(r) : "v"(sh), "v"(v));
    return r;
}
__device__ __forceinline__ uint32_t sdwa_shl_word1(uint32_t sh, uint32_t v)
{
    uint32_t r;
    asm volatile("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1"
        : "=v"(r) : "v"(sh), "v"(v));
    return r;
}

typedef float v4f __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------------
// M = 4 scan with conflict-free LDS reads ("subspace skew").
//
// TK = 32 centers per tile; 4 lanes form a slot and each lane owns 8 of the tile's centers (two
// 16-byte reads per subspace, the two halves of the 128-byte row), so a workgroup of T threads
// holds T/4 * R codes per tile fill.  Only the minimum over the lane's 8 centers and the tile
// index are tracked, so the order in which a lane meets its centers inside a tile does not matter.
// The tile image is x-major -- row (x, m) at byte x*512 + m*128 -- so that a row's LDS bank
// half is the parity of m and its quarter the half-row.  A 16-byte-per-lane LDS read is served
// 16 lanes = 4 slots per clock; the four slots of a group are made to hit four different bank
// quarters in every read: slots 0,1 of the group read subspace i in step i, slots 2,3 read
// subspace i-1 (one step behind); slots 0,2 take the lower half-row first, slots 1,3 the upper.
// The price of the skew is a fifth step per code: in the step a slot has no subspace to read it
// reads a line of -0.0 placed after the tile, and the sum becomes a chain of five terms
// (((V0 + V1) + V2) + V3) + V4 in which the -0.0 comes first or last.  Adding -0.0 returns the
// other operand bit for bit, so the value is exactly ((A0 + A1) + A2) + A3 in every lane.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float min3_f32(float a, float b, float c)
{
    float r;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

template <int R, int THREADS>
__global__ __launch_bounds__(THREADS) void assign_scan4s_kernel(const uint8_t* __restrict__ codes, int64_t N,
                                                                const float4* __restrict__ img, int ntiles,
                                                                int32_t* __restrict__ assign,
                                                                float* __restrict__ dist)
{
    constexpr int LPS = 4, TK = 32;
    constexpr int SLOTS = THREADS / LPS;
    constexpr int C = SLOTS * R;
    constexpr int NF = (TILE_F4 + THREADS - 1) / THREADS;     // float4 per thread per tile fill (last one partial)
    constexpr bool EVEN = TILE_F4 % THREADS == 0;
    constexpr uint32_t PAD = TILE_BYTES;      // 256 bytes of -0.0: [PAD, PAD+128) in bank half 0, the rest in half 1

    __shared__ float4 tile[TILE_F4 + 16];
    const char* tb = reinterpret_cast<const char*>(tile);

    const int tid = threadIdx.x;
    const int q = tid % LPS;
    const int c = tid / LPS;
    const uint32_t hsel = (uint32_t)c & 1u;           // odd slots start with the upper half-row
    const uint32_t late = ((uint32_t)c >> 1) & 1u;    // slots 2,3 of a group run one subspace behind
    const int64_t base = (int64_t)blockIdx.x * C;
    const uint32_t four = 4;

    if (tid < 16) tile[TILE_F4 + tid] = make_float4(-0.0f, -0.0f, -0.0f, -0.0f);

    // five step offsets per code, /16, in 16-bit fields: pa = f0|f1, pb = f2|f3; the fifth fields of
    // codes 2i and 2i+1 share pc[i]
    static_assert(R % 2 == 0, "fifth offsets are stored two to a register");
    uint32_t pa[R], pb[R], pc[R / 2];
    float best[R];
    int tix[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t n = base + (int64_t)r * SLOTS + c;
        if (n >= N) n = N - 1;
        uint32_t pk = *reinterpret_cast<const uint32_t*>(codes + n * 4);
        const uint32_t lo = (hsel << 2) | (uint32_t)q;                       // (hsel*64 + q*16) / 16
        uint32_t g0 = ((pk & 255u) << 5) | (0u << 3) | lo;                   // (x*512 + m*128)/16 = x*32 + m*8
        uint32_t g1 = (((pk >> 8) & 255u) << 5) | (1u << 3) | lo;
        uint32_t g2 = (((pk >> 16) & 255u) << 5) | (2u << 3) | lo;
        uint32_t g3 = ((pk >> 24) << 5) | (3u << 3) | lo;
        uint32_t dz = (PAD >> 4) + ((late ^ 1u) ? 0u : 8u) + lo;             // early slots pad in half 0, late ones in half 1
        uint32_t f0 = late ? dz : g0, f1 = late ? g0 : g1, f2 = late ? g1 : g2, f3 = late ? g2 : g3,
                 f4 = late ? g3 : dz;
        pa[r] = f0 | (f1 << 16);
        pb[r] = f2 | (f3 << 16);
        if (r & 1) pc[r / 2] |= f4 << 16; else pc[r / 2] = f4;
        best[r] = INFINITY;
        tix[r] = -1;
    }

    const uint32_t lane_off = (uint32_t)tid * 16u;
    v4f* ltile = reinterpret_cast<v4f*>(tile);
    auto gload = [&](int t, int i) -> v4f {
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float4*>(img + (size_t)t * TILE_F4), 0, TILE_BYTES, 0x00020000);
        return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, i * THREADS * 16, 0));
    };
    v4f pf[NF];
#pragma unroll
    for (int i = 0; i < NF; ++i) pf[i] = gload(0, i);

    struct Pair { float4 a, b; };
    auto issue = [&](int r, int i) -> Pair {
        uint32_t ad = (i == 0) ? sdwa_shl_word0(four, pa[r])
                    : (i == 1) ? sdwa_shl_word1(four, pa[r])
                    : (i == 2) ? sdwa_shl_word0(four, pb[r])
                    : (i == 3) ? sdwa_shl_word1(four, pb[r])
                    : (r & 1)  ? sdwa_shl_word1(four, pc[r / 2])
                               : sdwa_shl_word0(four, pc[r / 2]);
        Pair p;
        p.a = lds_read16(tb, ad);
        p.b = lds_read16(tb, ad ^ 64u);
        return p;
    };

    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NF; ++i)
            if (EVEN || i * THREADS + tid < TILE_F4) ltile[i * THREADS + tid] = pf[i];
        __syncthreads();
        {
            const int tn = t + 1 < ntiles ? t + 1 : t;
#pragma unroll
            for (int i = 0; i < NF; ++i) pf[i] = gload(tn, i);
        }
        Pair cur = issue(0, 0);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float4 sa, sb;
#pragma unroll
            for (int i = 0; i < 5; ++i) {
                Pair nxt = cur;
                if (i < 4) nxt = issue(r, i + 1);
                else if (r + 1 < R) nxt = issue(r + 1, 0);
                if (i == 0) {
                    sa = cur.a;
                    sb = cur.b;
                } else {
                    sa.x = sa.x + cur.a.x; sa.y = sa.y + cur.a.y; sa.z = sa.z + cur.a.z; sa.w = sa.w + cur.a.w;
                    sb.x = sb.x + cur.b.x; sb.y = sb.y + cur.b.y; sb.z = sb.z + cur.b.z; sb.w = sb.w + cur.b.w;
                }
                cur = nxt;
            }
            float m8 = __builtin_fminf(__builtin_fminf(sa.x, sa.y), sa.z);          // v_min3 chains
            m8 = __builtin_fminf(__builtin_fminf(m8, sa.w), sb.x);
            m8 = __builtin_fminf(__builtin_fminf(m8, sb.y), sb.z);
            m8 = __builtin_fminf(m8, sb.w);
            tix[r] = (m8 < best[r]) ? t : tix[r];
            best[r] = __builtin_fminf(best[r], m8);
        }
    }

    // Epilogue: recover the center inside the winning tile, then merge the 4 lanes of the slot.  Only lanes whose
    // minimum equals the slot's minimum can hold the winner, so only they re-read their sums' terms from the tile
    // image.  The four real subspace offsets are fields 0..3 (early slots) or 1..4 (late slots), and an offset is
    // the byte position inside the tile image.
    constexpr int G = THREADS > 768 ? 1 : (THREADS > 512 ? 2 : 4);
    static_assert(R % G == 0, "the epilogue handles codes in groups");
#pragma unroll 1
    for (int r0 = 0; r0 < R; r0 += G) {
        v4f w[G][8];
        float bq[G];
        int tq[G];
        bool need[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            uint32_t a = 0, b2 = 0, c2 = 0;
            bq[g] = INFINITY;
            tq[g] = -1;
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (r == r0 + g) { a = pa[r]; b2 = pb[r]; c2 = (r & 1) ? pc[r / 2] >> 16 : pc[r / 2]; tq[g] = tix[r]; bq[g] = best[r]; }
            float smin = bq[g];
#pragma unroll
            for (int d = LPS / 2; d >= 1; d >>= 1) smin = __builtin_fminf(smin, __shfl_xor(smin, d));
            need[g] = tq[g] >= 0 && bq[g] == smin;
#pragma unroll
            for (int i = 0; i < 8; ++i) w[g][i] = v4f{INFINITY, INFINITY, INFINITY, INFINITY};
            if (need[g]) {
                const char* gbase = reinterpret_cast<const char*>(img + (size_t)tq[g] * TILE_F4);
                const uint32_t e0 = a & 0xffffu, e1 = a >> 16, e2 = b2 & 0xffffu, e3 = b2 >> 16, e4 = c2 & 0xffffu;
                const uint32_t o0 = ((late ? e1 : e0) << 4) & ~64u, o1 = ((late ? e2 : e1) << 4) & ~64u;
                const uint32_t o2 = ((late ? e3 : e2) << 4) & ~64u, o3 = ((late ? e4 : e3) << 4) & ~64u;
                w[g][0] = *reinterpret_cast<const v4f*>(gbase + o0);
                w[g][1] = *reinterpret_cast<const v4f*>(gbase + o1);
                w[g][2] = *reinterpret_cast<const v4f*>(gbase + o2);
                w[g][3] = *reinterpret_cast<const v4f*>(gbase + o3);
                w[g][4] = *reinterpret_cast<const v4f*>(gbase + (o0 | 64u));
                w[g][5] = *reinterpret_cast<const v4f*>(gbase + (o1 | 64u));
                w[g][6] = *reinterpret_cast<const v4f*>(gbase + (o2 | 64u));
                w[g][7] = *reinterpret_cast<const v4f*>(gbase + (o3 | 64u));
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float b = INFINITY;
            int bi = IDX_NONE;
            v4f lo = w[g][0] + w[g][1];
            lo = lo + w[g][2];
            lo = lo + w[g][3];
            v4f hi = w[g][4] + w[g][5];
            hi = hi + w[g][6];
            hi = hi + w[g][7];
            if (need[g]) {
                const int kb = tq[g] * TK + q * 4;
                const float bb = bq[g];
                b = bb;
                if (hi.w == bb) { bi = kb + 19; b = hi.w; }
                if (hi.z == bb) { bi = kb + 18; b = hi.z; }
                if (hi.y == bb) { bi = kb + 17; b = hi.y; }
                if (hi.x == bb) { bi = kb + 16; b = hi.x; }
                if (lo.w == bb) { bi = kb + 3; b = lo.w; }
                if (lo.z == bb) { bi = kb + 2; b = lo.z; }
                if (lo.y == bb) { bi = kb + 1; b = lo.y; }
                if (lo.x == bb) { bi = kb; b = lo.x; }
            }
#pragma unroll
            for (int d = LPS / 2; d >= 1; d >>= 1) {
                float ob = __shfl_xor(b, d);
                int oi = __shfl_xor(bi, d);
                if (ob < b || (ob == b && oi < bi)) { b = ob; bi = oi; }
            }
            int64_t n = base + (int64_t)(r0 + g) * SLOTS + c;
            if (q == 0 && n < N) {
                assign[n] = (bi == IDX_NONE) ? 0 : bi;
                if (dist) dist[n] = b;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// ---------------------------------------------------------------------------------------------
// Regrouping of M = 4 codes for the conflict-free scans below.
//
// A ds_read_b128 is served 16 lanes per clock, and on gfx950 those are lanes {0-3, 12-15, 20-23,
// 24-27} and {4-7, 8-11, 16-19, 28-31} of each half-wave: with 4 lanes per code ("slot") the
// slots {0, 3, 5, 6} and {1, 2, 4, 7} of every aligned block of 8 slots are served together
// (measured: the bank-conflict counter reads zero only for this partition).  Such a set of four
// codes reads conflict-free in all four subspaces when, in every subspace, the four subcodes are
// different mod 4 -- a "residue group".
//
// The class of a code is its four residues as one byte (256 classes).  Take two class-valued
// masks a, b whose 2-bit fields are non-zero and different in every subspace: the classes
// c, c^a, c^b, c^a^b (an orbit) then differ in every subspace, so one code from each is a residue
// group, and the residue of subspace 0 serves as the code's slot in it.  The plan goes through
// GROUP_ROUNDS such mask pairs and takes, from every orbit, as many groups as its rarest class
// still has; what no round can match is left over and put in groups of four as it comes.
// Left-over groups are spread evenly between the residue groups so that every workgroup gets its
// share of their bank conflicts.
//
// Three launches: per-workgroup class histograms, the plan (one workgroup), the scatter.  The
// count and scatter kernels split the codes the same way, so the plan can hand every scatter
// workgroup its first rank in every class and the result is deterministic.
//
// Nothing here affects results: the scan treats every code independently, and writes each result
// to the code's original position.
// ---------------------------------------------------------------------------------------------
constexpr uint32_t ORIGIN_NONE = 0xffffffffu;   // a position of the regrouped array that holds no code
constexpr int GROUP_ROUNDS = 16;
constexpr int GROUP_MAX_WGS = 256;              // workgroups of the count and scatter kernels
constexpr int GROUP_THREADS = 1024;

__constant__ uint8_t group_masks[GROUP_ROUNDS][2] = {
    {0x7b, 0xae}, {0x66, 0x9b}, {0x69, 0xb7}, {0x7d, 0xaa}, {0x7b, 0x96}, {0x57, 0xbe}, {0x6f, 0xb5}, {0x77, 0x9a},
    {0x6f, 0xb9}, {0x6d, 0xb7}, {0x5a, 0xa7}, {0x5d, 0xa6}, {0x5d, 0xaa}, {0x67, 0xb9}, {0x6d, 0x97}, {0x57, 0xae}};

struct GroupPlan {
    uint32_t first[256][GROUP_ROUNDS + 1];   // per class: rank of its first code matched in round d; [last] = all matched
    uint32_t gbase[256][GROUP_ROUNDS];       // per class: index of the first group its orbit forms in round d
    uint32_t lbase[256];                     // per class: index of its first left-over code among all left-overs
    uint32_t groups, leftovers, lgroups, period_m1;   // residue groups, left-over codes, their groups of 4, D-1
    uint32_t wg_hist[GROUP_MAX_WGS][256];    // count pass: codes per (workgroup, class); then the workgroup's first rank
};

__device__ __forceinline__ uint32_t code_class(uint32_t pk)
{
    return (pk & 3u) | ((pk >> 6) & 0xcu) | ((pk >> 12) & 0x30u) | ((pk >> 18) & 0xc0u);
}

// The codes left over by the matching are dealt to groups by quarters of their list: member k of a left-over group
// is the code at the same place of quarter k.  The list is therefore ordered by a key under which, if the quarters are
// balanced, codes at the same place of different quarters differ mod 4 in every subspace: the top digit (2 bits) is
// the residue of the last subspace, every other digit that subspace's residue plus the top digit, mod 4.  The deeper
// a digit, the sooner uneven class sizes put the quarters out of step; the first few subspaces are what is gained.
// This is the key's inverse: the class (2 bits per subspace) that holds place `key` of the order.
__device__ __forceinline__ uint32_t leftover_order_class(uint32_t key, int nsub)
{
    const uint32_t top = key >> (2 * (nsub - 1));
    uint32_t c = top << (2 * (nsub - 1));
    for (int s = 0; s < nsub - 1; ++s) c |= (((key >> (2 * s)) - top) & 3u) << (2 * s);
    return c;
}

// Place of residue group g / of left-over group jg in the final order of all groups (gtot residue groups, lg left-over
// groups, dm1 = gtot / lg).  The left-over groups are spread evenly among the residue groups, so that every workgroup
// gets its share of their bank conflicts: one after every dm1 residue groups for the four-lane scans; for the
// two-lane scans, whose LDS accesses hold the groups 2i and 2i + 1 together, two after every 2 dm1 (pairs != 0): two
// left-over groups that share their accesses cost about the conflicts of one.
__device__ __forceinline__ int64_t residue_group_place(uint32_t g, uint32_t lg, uint32_t dm1, int pairs)
{
    if (!dm1) return g;
    if (!pairs) {
        const uint32_t before = g / dm1;
        return (int64_t)g + (before < lg ? before : lg);
    }
    const uint32_t before = 2u * (g / (2u * dm1)), all = lg & ~1u;
    return (int64_t)g + (before < all ? before : all);
}
__device__ __forceinline__ int64_t leftover_group_place(uint32_t jg, uint32_t gtot, uint32_t lg, uint32_t dm1, int pairs)
{
    if (!dm1) return (int64_t)gtot + jg;
    if (!pairs) return (int64_t)jg * (dm1 + 1) + dm1;
    if (jg < (lg & ~1u)) return (int64_t)(jg >> 1) * (2 * dm1 + 2) + 2 * dm1 + (jg & 1u);
    return (int64_t)gtot + lg - 1;                  // an odd one out closes the list
}

// position of slot `slot` of group `u` (counting residue and left-over groups in their final order): groups
// 2b and 2b+1 share the block of 8 slots b and take the slots the LDS serves together
__device__ __forceinline__ int64_t group_slot_position(int64_t u, uint32_t slot)
{
    const uint32_t even_slots = 0x6530u, odd_slots = 0x7421u;      // {0,3,5,6} and {1,2,4,7}, 4 bits each
    const uint32_t map = (u & 1) ? odd_slots : even_slots;
    return (u >> 1) * 8 + ((map >> (4 * slot)) & 15u);
}

// The same for the scan whose slots are two lanes wide (assign_scan4q_kernel): an LDS access then serves eight
// slots, {0,1,6,7,10,11,12,13} or {2,3,4,5,8,9,14,15} of a block of 16, of which the even ones read the lower
// half of their row first and the odd ones the upper: four groups share a block, group 4b + g takes the slots
// {0,6,10,12}, {1,7,11,13}, {2,4,8,14}, {3,5,9,15}.
__device__ __forceinline__ int64_t group_slot_position16(int64_t u, uint32_t slot)
{
    const uint32_t maps[4] = {0xca60u, 0xdb71u, 0xe842u, 0xf953u};
    return (u >> 2) * 16 + ((maps[u & 3] >> (4 * slot)) & 15u);
}

// gco[pos] = (0, ORIGIN_NONE) for every position: the two-lane-slot layout marks its holes this way before the scatter
__global__ __launch_bounds__(256) void code_group_clear_kernel(uint2* __restrict__ gco, int64_t n_alloc)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_alloc; i += (int64_t)gridDim.x * 256)
        gco[i] = make_uint2(0u, 0xffffffffu);
}

// Workgroup w of gridDim.x takes the chunks of 1024 consecutive codes w, w + gridDim.x, ...
__global__ __launch_bounds__(GROUP_THREADS) void code_class_count_kernel(const uint8_t* __restrict__ codes, int64_t n,
                                                                         GroupPlan* __restrict__ plan)
{
    __shared__ uint32_t h[256];
    if (threadIdx.x < 256) h[threadIdx.x] = 0u;
    __syncthreads();
    const uint32_t* cw = reinterpret_cast<const uint32_t*>(codes);
    for (int64_t i = (int64_t)blockIdx.x * GROUP_THREADS + threadIdx.x; i < n; i += (int64_t)gridDim.x * GROUP_THREADS)
        atomicAdd(&h[code_class(cw[i])], 1u);
    __syncthreads();
    if (threadIdx.x < 256) plan->wg_hist[blockIdx.x][threadIdx.x] = h[threadIdx.x];
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t o = __shfl_up(v, off);
        if ((int)(threadIdx.x & 63) >= off) v += o;
    }
    return v;
}

// one workgroup of 1024 threads; nwg <= GROUP_MAX_WGS = workgroups of the count pass
__global__ __launch_bounds__(1024) void code_group_plan_kernel(GroupPlan* __restrict__ plan, int nwg)
{
    __shared__ uint32_t part[4][256];
    __shared__ uint32_t tot[256];
    __shared__ uint32_t rem[256];
    const int tid = threadIdx.x;
    // --- class totals and every workgroup's first rank: thread (p, c) owns rows [p*rows, (p+1)*rows) of class c,
    //     all of them loaded before the first is used
    {
        constexpr int ROWS_MAX = GROUP_MAX_WGS / 4;
        const int p = tid >> 8, c = tid & 255;
        const int rows = (nwg + 3) / 4;
        const int w0 = p * rows;
        // buffer addressing: one lane offset, the row as a constant offset -- no address registers per row.  Rows
        // up to 4*rows - 1 <= 255 exist in the array; those past nwg hold nothing and are masked.
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(&plan->wg_hist[0][0], 0,
                                                                      GROUP_MAX_WGS * 256 * 4, 0x00020000);
        const uint32_t lane_off = (uint32_t)(w0 * 256 + c) * 4u;
        uint32_t v[ROWS_MAX];
#pragma unroll
        for (int k = 0; k < ROWS_MAX; ++k) v[k] = __builtin_amdgcn_raw_buffer_load_b32(rs, lane_off, k * 1024, 0);
        uint32_t sum = 0;
#pragma unroll
        for (int k = 0; k < ROWS_MAX; ++k) {
            if (!(k < rows && w0 + k < nwg)) v[k] = 0u;
            sum += v[k];
        }
        part[p][c] = sum;
        __syncthreads();
        uint32_t run = 0;
        for (int pp = 0; pp < p; ++pp) run += part[pp][c];
#pragma unroll
        for (int k = 0; k < ROWS_MAX; ++k) {
            // lanes whose row is not theirs point past the end of the buffer, where stores are dropped
            const uint32_t off = (k < rows) ? lane_off : 0x7ffffff0u;
            __builtin_amdgcn_raw_buffer_store_b32(run, rs, off, k * 1024, 0);
            run += v[k];
        }
        if (p == 0) {
            const uint32_t t = part[0][c] + part[1][c] + part[2][c] + part[3][c];
            tot[c] = t;
            rem[c] = t;
        }
        __syncthreads();
    }
    if (tid >= 64) return;           // no barrier below: the matching runs in one wave
    // --- lane j owns, in every round, the orbit led by class 4j (residue 0 in subspace 0): every class is in
    //     exactly one orbit per round, so the lanes never touch the same entry of rem
    //     First all rounds' group counts (a dependent chain through rem), then the prefix sums of all rounds
    //     (independent of each other, so their cross-lane steps overlap).
    uint32_t mm[GROUP_ROUNDS];
#pragma unroll
    for (int d = 0; d < GROUP_ROUNDS; ++d) {
        const uint32_t a = group_masks[d][0], b = group_masks[d][1];
        const uint32_t c0 = (uint32_t)tid << 2, c1 = c0 ^ a, c2 = c0 ^ b, c3 = c0 ^ a ^ b;
        const uint32_t r0 = rem[c0], r1 = rem[c1], r2 = rem[c2], r3 = rem[c3];
        uint32_t m = r0 < r1 ? r0 : r1;
        m = m < r2 ? m : r2;
        m = m < r3 ? m : r3;
        mm[d] = m;
        plan->first[c0][d] = tot[c0] - r0;
        plan->first[c1][d] = tot[c1] - r1;
        plan->first[c2][d] = tot[c2] - r2;
        plan->first[c3][d] = tot[c3] - r3;
        rem[c0] = r0 - m;  rem[c1] = r1 - m;  rem[c2] = r2 - m;  rem[c3] = r3 - m;
        // one wave: its LDS accesses complete in program order, so the next round reads these values; the
        // compiler keeps the order because the indices may alias
        __builtin_amdgcn_wave_barrier();
    }
    uint32_t gtot = 0;
#pragma unroll
    for (int d = 0; d < GROUP_ROUNDS; ++d) {
        const uint32_t a = group_masks[d][0], b = group_masks[d][1];
        const uint32_t c0 = (uint32_t)tid << 2, c1 = c0 ^ a, c2 = c0 ^ b, c3 = c0 ^ a ^ b;
        const uint32_t inc = wave_inclusive_scan(mm[d]);
        const uint32_t base = gtot + inc - mm[d];
        gtot += __shfl(inc, 63);
        plan->gbase[c0][d] = base;
        plan->gbase[c1][d] = base;
        plan->gbase[c2][d] = base;
        plan->gbase[c3][d] = base;
    }
    // --- left-overs: exclusive prefix over the classes in the order of leftover_order_class, lane j owns places
    //     4j .. 4j+3 of it
    {
        const uint32_t k0 = (uint32_t)tid << 2;
        const uint32_t c0 = leftover_order_class(k0, 4), c1 = leftover_order_class(k0 + 1, 4),
                       c2 = leftover_order_class(k0 + 2, 4), c3 = leftover_order_class(k0 + 3, 4);
        const uint32_t l0 = rem[c0], l1 = rem[c1], l2 = rem[c2], l3 = rem[c3];
        const uint32_t mine = l0 + l1 + l2 + l3;
        const uint32_t inc = wave_inclusive_scan(mine);
        uint32_t e = inc - mine;
        plan->first[c0][GROUP_ROUNDS] = tot[c0] - l0;  plan->lbase[c0] = e;  e += l0;
        plan->first[c1][GROUP_ROUNDS] = tot[c1] - l1;  plan->lbase[c1] = e;  e += l1;
        plan->first[c2][GROUP_ROUNDS] = tot[c2] - l2;  plan->lbase[c2] = e;  e += l2;
        plan->first[c3][GROUP_ROUNDS] = tot[c3] - l3;  plan->lbase[c3] = e;
        if (tid == 63) {
            const uint32_t ltot = inc, lg = (ltot + 3u) / 4u;
            plan->groups = gtot;
            plan->leftovers = ltot;
            plan->lgroups = lg;
            plan->period_m1 = (lg > 0 && gtot >= lg) ? gtot / lg : 0u;   // D-1 residue groups between two left-over groups
        }
    }
}

// gco[pos] = (code, original index); positions that receive no code get (0, ORIGIN_NONE)
__global__ __launch_bounds__(GROUP_THREADS) void code_group_scatter_kernel(const uint8_t* __restrict__ codes, int64_t n,
                                                                           const GroupPlan* __restrict__ plan,
                                                                           uint2* __restrict__ gco, int64_t n_alloc,
                                                                           int blocks_of_16 = 0)
{
    __shared__ uint32_t cur[256];
    __shared__ uint32_t first_s[256][GROUP_ROUNDS + 1];
    __shared__ uint32_t gbase_s[256][GROUP_ROUNDS];
    __shared__ uint32_t lbase_s[256];
    const int tid = threadIdx.x;
    if (tid < 256) {
        cur[tid] = plan->wg_hist[blockIdx.x][tid];
        lbase_s[tid] = plan->lbase[tid];
    }
    for (int i = tid; i < 256 * (GROUP_ROUNDS + 1); i += GROUP_THREADS) (&first_s[0][0])[i] = (&plan->first[0][0])[i];
    for (int i = tid; i < 256 * GROUP_ROUNDS; i += GROUP_THREADS) (&gbase_s[0][0])[i] = (&plan->gbase[0][0])[i];
    const uint32_t gtot = plan->groups, ltot = plan->leftovers, lg = plan->lgroups, dm1 = plan->period_m1;
    __syncthreads();
    const uint32_t* cw = reinterpret_cast<const uint32_t*>(codes);
    for (int64_t i = (int64_t)blockIdx.x * GROUP_THREADS + tid; i < n; i += (int64_t)gridDim.x * GROUP_THREADS) {
        const uint32_t pk = cw[i];
        const uint32_t c = code_class(pk);
        const uint32_t rank = atomicAdd(&cur[c], 1u);
        int64_t u;
        uint32_t slot;
        if (rank < first_s[c][GROUP_ROUNDS]) {
            int d = 0;
            if (rank >= first_s[c][1]) {              // most codes are matched in the first round
#pragma unroll
                for (int e = 1; e < GROUP_ROUNDS; ++e)
                    if (rank >= first_s[c][e]) d = e;
            }
            const uint32_t g = gbase_s[c][d] + (rank - first_s[c][d]);
            slot = c & 3u;
            u = residue_group_place(g, lg, dm1, blocks_of_16);
        } else {
            // left-overs come in the order of leftover_order_class: group j takes the left-overs j, j + lg, j + 2 lg,
            // j + 3 lg, four different stretches of that order, rather than four neighbours of (mostly) one class
            const uint32_t li = lbase_s[c] + (rank - first_s[c][GROUP_ROUNDS]);
            const uint32_t jg = li % lg;
            slot = li / lg;
            u = leftover_group_place(jg, gtot, lg, dm1, blocks_of_16);
        }
        const int64_t pos = blocks_of_16 ? group_slot_position16(u, slot) : group_slot_position(u, slot);
        if (pos < n_alloc) gco[pos] = make_uint2(pk, (uint32_t)i);
    }
    // holes: the empty places of the left-over groups, the second half of the last block of 8, the tail
    // (blocks of 16: every position was marked empty before this kernel ran)
    if (blockIdx.x == 0 && tid < 32 && !blocks_of_16) {
        const int64_t T = (int64_t)gtot + lg;
        int64_t pos = -1;
        if (tid < 4) {
            // the left-over groups have 4 lg >= ltot places: the places ltot .. 4 lg - 1 (at most 3) stay empty
            const uint32_t li = ltot + (uint32_t)tid;
            if (li < 4u * lg) {
                const uint32_t jg = li % lg;
                pos = group_slot_position(leftover_group_place(jg, gtot, lg, dm1, 0), li / lg);
            }
        } else if (tid < 8) {
            if (T & 1) pos = group_slot_position(T, (uint32_t)tid - 4);
        } else {
            pos = ((T + 1) >> 1) * 8 + (tid - 8);
        }
        if (pos >= 0 && pos < n_alloc) gco[pos] = make_uint2(0u, ORIGIN_NONE);
    }
}

// ---------------------------------------------------------------------------------------------
// M = 4 scan over residue-grouped codes ("half-plane" tile image).
//
// Same decomposition as assign_scan4s_kernel (4 lanes per slot, 8 centers per lane, TK = 32),
// but the tile image is stored as eight planes, one per (subspace m, half h of the tile's
// centers): the 64 bytes of centers 16h .. 16h+15 for subcode x sit at byte
//      (2m + h) * 16384 + x * 64,
// so the 64-byte bank quarter a slot reads is x mod 4 in every one of its eight reads, and both
// halves of all four rows are reached from four per-code offsets through the instruction's
// immediate offset: no address arithmetic beyond unpacking one 16-bit field per subspace, no
// skew step, 3 adds per evaluation.  A 16-byte-per-lane LDS read is served 16 lanes = 4 slots per
// clock, so it is conflict-free exactly when the four codes of a slot group have four different
// subcodes mod 4 in that subspace.  Any order of the codes gives the same result; the order only
// decides the speed.  The caller therefore passes the codes regrouped so that as many aligned
// groups of four as possible have that property in all four subspaces (code_group_* kernels
// below) as (code, original index) pairs; the result is written to the original index.
// ---------------------------------------------------------------------------------------------
// What the scan leaves for the histogram pass when BUCKET is set: workgroup w files its codes by cluster group
// (KT consecutive clusters) into its own stretch [w*C, (w+1)*C) of `pool` as (code, center) records, the groups
// one after the other, and notes (first record, number of records) of group g in seg[g * gridDim.x + w].
// What a scan leaves for the sorted-path histogram when `count` is set: count[k] is incremented for every code
// assigned to center k (it must be zero before the first scan launch of the assignment step) and rank[n] receives
// the value the increment returned, the code's place among the members of its cluster.  With the exclusive prefix
// of the counts that is the code's position in the order by cluster: no counting pass over the assignments and no
// atomics in the scatter.
struct RankOut {
    uint32_t* count = nullptr;
    uint32_t* rank = nullptr;
};

struct BucketOut {
    uint2* pool;
    uint2* seg;
    int KT;          // clusters per group
    int ngroups;     // at most 256
};

template <int R, int THREADS, int DEPTH, bool BUCKET = false>
__global__ __launch_bounds__(THREADS) void assign_scan4p_kernel(const uint8_t* __restrict__ codes, int64_t N,
                                                                const uint2* __restrict__ gco,
                                                                const float4* __restrict__ img,
                                                                const float4* __restrict__ rows, int ntiles,
                                                                int32_t* __restrict__ assign,
                                                                float* __restrict__ dist, BucketOut bo,
                                                                RankOut ro = RankOut{})
{
    constexpr int LPS = 4, TK = 32;
    constexpr int SLOTS = THREADS / LPS;
    constexpr int C = SLOTS * R;
    constexpr int NF = (TILE_F4 + THREADS - 1) / THREADS;     // float4 per thread per tile fill (last one partial)
    constexpr bool EVEN = TILE_F4 % THREADS == 0;
    constexpr uint32_t HPLANE = 16384;      // bytes per (m, h) plane: 256 subcodes x 16 centers

    __shared__ float4 tile[TILE_F4];
    __shared__ uint32_t gcnt[BUCKET ? 256 : 1], gbase[BUCKET ? 256 : 1];   // codes per cluster group, first record
    const char* tb = reinterpret_cast<const char*>(tile);

    const int tid = threadIdx.x;
    const int q = tid % LPS;
    const int c = tid / LPS;
    const int64_t base = (int64_t)blockIdx.x * C;
    const uint32_t low15 = 0x7fffu;
    if (BUCKET && tid < 256) gcnt[tid] = 0u;       // the tile loop's barriers come before its first use

    // per code two registers, each a 15-bit and a 17-bit field: the byte offset of the lane's piece in its row
    // (subspaces 0 and 1, low fields) and the same plus 64 KB (subspaces 2 and 3, high fields), so that every
    // remaining plane offset (0 to 3 planes of 16 KB) fits the DS immediate and each unpack is one full-rate op
    uint32_t pa[R], pb[R];
    float best[R];
    int tix[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t n = base + (int64_t)r * SLOTS + c;
        if (n >= N) n = N - 1;
        uint32_t pk = gco ? gco[n].x : *reinterpret_cast<const uint32_t*>(codes + n * 4);
        uint32_t f0 = ((pk & 255u) << 6) | ((uint32_t)q << 4);
        uint32_t f1 = (((pk >> 8) & 255u) << 6) | ((uint32_t)q << 4);
        uint32_t f2 = ((((pk >> 16) & 255u) << 6) | ((uint32_t)q << 4)) + 65536u;
        uint32_t f3 = (((pk >> 24) << 6) | ((uint32_t)q << 4)) + 65536u;
        pa[r] = f0 | (f2 << 15);
        pb[r] = f1 | (f3 << 15);
        best[r] = INFINITY;
        tix[r] = -1;
    }

    const uint32_t lane_off = (uint32_t)tid * 16u;
    v4f* ltile = reinterpret_cast<v4f*>(tile);
    auto gload = [&](int t, int i) -> v4f {
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float4*>(img + (size_t)t * TILE_F4), 0, TILE_BYTES, 0x00020000);
        return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, i * THREADS * 16, 0));
    };
    v4f pf[NF];
#pragma unroll
    for (int i = 0; i < NF; ++i) pf[i] = gload(0, i);

    // A step is one subspace of one code: two 16-byte reads (the two halves of the tile's centers).  The
    // reads of the next DEPTH steps are in flight while the sums of the current one are formed: with
    // 16-byte reads the LDS pipe needs several outstanding per wave to stay busy next to the adds.
    struct Pair { float4 a, b; };
    auto issue = [&](int step) -> Pair {
        const int r = step / 4, m = step % 4;
        uint32_t ad = (m == 0) ? unpack_low15(low15, pa[r])
                    : (m == 1) ? unpack_low15(low15, pb[r])
                    : (m == 2) ? unpack_high17(pa[r])
                               : unpack_high17(pb[r]);
        const uint32_t po = (m & 1) ? 2 * HPLANE : 0;
        Pair p;
        p.a = lds_read16(tb, ad + po);
        p.b = lds_read16(tb, ad + po + HPLANE);
        return p;
    };

    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NF; ++i)
            if (EVEN || i * THREADS + tid < TILE_F4) ltile[i * THREADS + tid] = pf[i];
        __syncthreads();
        // the loads of the next tile are spread over the first 5/8 of the scan: issued in one burst they
        // would keep every wave in the vector-memory issue queue while the LDS pipe idles
        const int tn = t + 1 < ntiles ? t + 1 : t;
        Pair ring[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) ring[d] = issue(d);
        float4 sa, sb;
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int i = 0; i < NF; ++i)
                if ((i * R * 5) / (NF * 8) == r) pf[i] = gload(tn, i);
#pragma unroll
          for (int m = 0; m < 4; ++m) {
            const int step = 4 * r + m;
            const Pair cur = ring[step % DEPTH];
            if (step + DEPTH < 4 * R) ring[step % DEPTH] = issue(step + DEPTH);
            if (m == 0) {
                sa = cur.a;
                sb = cur.b;
            } else {
                sa.x = sa.x + cur.a.x; sa.y = sa.y + cur.a.y; sa.z = sa.z + cur.a.z; sa.w = sa.w + cur.a.w;
                sb.x = sb.x + cur.b.x; sb.y = sb.y + cur.b.y; sb.z = sb.z + cur.b.z; sb.w = sb.w + cur.b.w;
            }
            if (m == 3) {
                float m8 = min3_f32(sa.x, sa.y, sa.z);
                m8 = min3_f32(m8, sa.w, sb.x);
                m8 = min3_f32(m8, sb.y, sb.z);
                const float nb = min3_f32(m8, sb.w, best[r]);
                tix[r] = (nb < best[r]) ? t : tix[r];
                best[r] = nb;
            }
          }
        }
    }

    // Epilogue: recover the center inside the winning tile.  During the scan four lanes share a code; here the
    // work is transposed through LDS so that every lane finishes codes of its own (R/4 of them) instead of four
    // lanes walking through the same R codes: each lane leaves (minimum, tile) per code in LDS, then lane l takes
    // the codes l, l + THREADS, ...: the slot minimum is the smallest of the four minima, the winning tile the
    // lowest tile among the lanes that attain it (a lower tile means lower center indices), and for every lane
    // position q that attains it in that tile the 8 sums of its centers are rebuilt from the tile image in global
    // memory (same bits, same sum order) and the lowest center index with that sum is kept.  Almost always there
    // is one such q; the loop over them only repeats on exact ties between lane positions.
    static_assert(R * THREADS * 8 <= TILE_BYTES, "the per-lane records must fit the tile buffer");
    constexpr int CPL = (R + 3) / 4;                // codes per lane in the epilogue (the last ones may be past C)
    constexpr int EB = THREADS > 768 ? 2 : 4;       // codes whose image reads are in flight together
    __syncthreads();                                // every wave is done with the last tile
    {
        float2* rec = reinterpret_cast<float2*>(tile);
#pragma unroll
        for (int r = 0; r < R; ++r)                  // record index = 4 * (code index in the workgroup) + q
            rec[(r * SLOTS + c) * 4 + q] = make_float2(best[r], __builtin_bit_cast(float, tix[r]));
    }
    __syncthreads();
    // The reads go to the copy of the images in the order [tile][m][x][32 centers]: the 8 pieces of a code are
    // then in 4 cache lines instead of 8 (a scattered 16-byte read moves a whole 128-byte line, and this traffic
    // is what the epilogue costs).  The whole copy sits behind one buffer descriptor (the host uses this kernel
    // only while it is below 4 GB): a 32-bit lane offset per subspace, the subspace plane as a scalar offset;
    // offsets past the end return zero.
    __amdgpu_buffer_rsrc_t rs_img = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float4*>(rows), 0, (uint32_t)ntiles * (uint32_t)TILE_BYTES, 0x00020000);
    constexpr int TNONE = 0x7fffffff;
#pragma unroll 1
    for (int i0 = 0; i0 < CPL; i0 += EB) {
        float smin[EB];
        int tmin[EB], bi[EB];
        uint32_t cand[EB], pk[EB], og[EB];
        v4f w[EB][8];
        int qq[EB];
        // phase A: records, code, original position
#pragma unroll
        for (int e = 0; e < EB; ++e) {
            if (i0 + e >= CPL) { cand[e] = 0u; og[e] = ORIGIN_NONE; pk[e] = 0u; smin[e] = 0.f; tmin[e] = 0; bi[e] = IDX_NONE; continue; }
            const int j = (i0 + e) * THREADS + tid;
            int64_t n = base + j;
            const bool live = n < N && j < C;
            if (!live) n = N - 1;
            const float4 ra = lds_read16(tb, (uint32_t)j * 32u), rb = lds_read16(tb, (uint32_t)j * 32u + 16u);
            const float b0 = ra.x, b1 = ra.z, b2 = rb.x, b3 = rb.z;
            const int t0 = __builtin_bit_cast(int, ra.y), t1 = __builtin_bit_cast(int, ra.w);
            const int t2 = __builtin_bit_cast(int, rb.y), t3 = __builtin_bit_cast(int, rb.w);
            const float sm = __builtin_fminf(__builtin_fminf(b0, b1), __builtin_fminf(b2, b3));
            const int c0 = (b0 == sm && t0 >= 0) ? t0 : TNONE, c1 = (b1 == sm && t1 >= 0) ? t1 : TNONE;
            const int c2 = (b2 == sm && t2 >= 0) ? t2 : TNONE, c3 = (b3 == sm && t3 >= 0) ? t3 : TNONE;
            int tm = c0 < c1 ? c0 : c1;
            tm = tm < c2 ? tm : c2;
            tm = tm < c3 ? tm : c3;
            uint32_t cd = (uint32_t)(c0 == tm) | ((uint32_t)(c1 == tm) << 1) | ((uint32_t)(c2 == tm) << 2) |
                          ((uint32_t)(c3 == tm) << 3);
            if (tm == TNONE || !live) cd = 0u;
            smin[e] = sm;
            tmin[e] = tm;
            cand[e] = cd;
            bi[e] = IDX_NONE;
            if (gco) {
                const uint2 g = gco[n];
                pk[e] = g.x;
                og[e] = live ? g.y : ORIGIN_NONE;
            } else {
                pk[e] = *reinterpret_cast<const uint32_t*>(codes + n * 4);
                og[e] = live ? 0u : ORIGIN_NONE;
            }
        }
        // phase B: lowest candidate position of every code, all reads in flight together; then any further
        // candidates (exact ties between lane positions), one at a time
        auto ep_issue = [&](int e) {
            const uint32_t cd = cand[e];
            const int qe = cd ? (int)__builtin_ctz(cd) : 0;
            qq[e] = qe;
            const uint32_t tb0 = cd ? (uint32_t)tmin[e] * (uint32_t)TILE_BYTES + (uint32_t)qe * 16u : 0xfff00000u;
            const uint32_t o0 = tb0 + ((pk[e] & 255u) << 7), o1 = tb0 + (((pk[e] >> 8) & 255u) << 7);
            const uint32_t o2 = tb0 + (((pk[e] >> 16) & 255u) << 7), o3 = tb0 + ((pk[e] >> 24) << 7);
            constexpr int MP = 32768;             // bytes per subspace in a tile of the row copy
            w[e][0] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o0, 0, 0));
            w[e][4] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o0, 64, 0));
            w[e][1] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o1, MP, 0));
            w[e][5] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o1, MP + 64, 0));
            w[e][2] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o2, 2 * MP, 0));
            w[e][6] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o2, 2 * MP + 64, 0));
            w[e][3] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o3, 3 * MP, 0));
            w[e][7] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o3, 3 * MP + 64, 0));
        };
        auto ep_finish = [&](int e) {
            if (cand[e]) {
                v4f lo = w[e][0] + w[e][1];
                lo = lo + w[e][2];
                lo = lo + w[e][3];
                v4f hi = w[e][4] + w[e][5];
                hi = hi + w[e][6];
                hi = hi + w[e][7];
                const int kb = tmin[e] * TK + qq[e] * 4;
                const float bb = smin[e];
                int k = IDX_NONE;
                if (hi.w == bb) k = kb + 19;
                if (hi.z == bb) k = kb + 18;
                if (hi.y == bb) k = kb + 17;
                if (hi.x == bb) k = kb + 16;
                if (lo.w == bb) k = kb + 3;
                if (lo.z == bb) k = kb + 2;
                if (lo.y == bb) k = kb + 1;
                if (lo.x == bb) k = kb;
                bi[e] = k < bi[e] ? k : bi[e];
                cand[e] &= cand[e] - 1u;
            }
        };
        // one trip handles the lowest candidate position of every code of the batch; further trips only happen
        // on exact ties between lane positions (the loop is one copy of the code: this part of the kernel runs
        // once per workgroup, from a cold instruction cache, and its size is its cost)
        bool more;
        do {
#pragma unroll
            for (int e = 0; e < EB; ++e) ep_issue(e);
#pragma unroll
            for (int e = 0; e < EB; ++e) ep_finish(e);
            more = false;
#pragma unroll
            for (int e = 0; e < EB; ++e) more = more || cand[e] != 0u;
        } while (__any(more));
#pragma unroll
        for (int e = 0; e < EB; ++e) {
            if (og[e] != ORIGIN_NONE) {
                const int64_t dst = gco ? (int64_t)og[e] : base + (i0 + e) * THREADS + tid;
                const int kw = (bi[e] == IDX_NONE) ? 0 : bi[e];
                assign[dst] = kw;
                if (dist) dist[dst] = smin[e];
                if (ro.count) ro.rank[dst] = atomicAdd(&ro.count[kw], 1u);
            }
            if (BUCKET && i0 + e < CPL) {
                // the code's 32-byte slot of records has been read (by this lane only): it now keeps the code, its
                // center, its cluster group and its rank among the workgroup's codes of that group
                const uint32_t k = (bi[e] == IDX_NONE) ? 0u : (uint32_t)bi[e];
                uint32_t g = 0xffffffffu, rank = 0u;
                if (og[e] != ORIGIN_NONE) {
                    g = k / (uint32_t)bo.KT;
                    g = g < 255u ? g : 255u;                     // k < K and at most 255 groups: never taken
                    rank = atomicAdd(&gcnt[g], 1u);
                }
                const int j = (i0 + e) * THREADS + tid;
                *reinterpret_cast<uint4*>(reinterpret_cast<char*>(tile) + (size_t)j * 32u) = make_uint4(pk[e], k, g, rank);
            }
        }
    }
    if (BUCKET) {
        __syncthreads();
        if (tid < 64) {                                          // exclusive prefix over the groups: lane l owns 4l .. 4l+3
            const uint32_t a0 = gcnt[4 * tid], a1 = gcnt[4 * tid + 1], a2 = gcnt[4 * tid + 2], a3 = gcnt[4 * tid + 3];
            const uint32_t mine = a0 + a1 + a2 + a3;
            const uint32_t e0 = wave_inclusive_scan(mine) - mine, e1 = e0 + a0, e2 = e1 + a1, e3 = e2 + a2;
            gbase[4 * tid] = e0;  gbase[4 * tid + 1] = e1;  gbase[4 * tid + 2] = e2;  gbase[4 * tid + 3] = e3;
            const size_t nw = gridDim.x;
            uint2* sg = bo.seg + blockIdx.x;
            if (4 * tid < bo.ngroups) sg[(size_t)(4 * tid) * nw] = make_uint2((uint32_t)(base + e0), a0);
            if (4 * tid + 1 < bo.ngroups) sg[(size_t)(4 * tid + 1) * nw] = make_uint2((uint32_t)(base + e1), a1);
            if (4 * tid + 2 < bo.ngroups) sg[(size_t)(4 * tid + 2) * nw] = make_uint2((uint32_t)(base + e2), a2);
            if (4 * tid + 3 < bo.ngroups) sg[(size_t)(4 * tid + 3) * nw] = make_uint2((uint32_t)(base + e3), a3);
        }
        __syncthreads();
#pragma unroll 1
        for (int i = 0; i < CPL; ++i) {
            const int j = i * THREADS + tid;
            const uint4 r = *reinterpret_cast<const uint4*>(tb + (size_t)j * 32u);
            if (r.z != 0xffffffffu) bo.pool[base + gbase[r.z] + r.w] = make_uint2(r.x, r.y);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Inputs of the table-built tiles (see TileSource): tabT[m][c][x] = tables[m][x][c] with one extra row of +inf, and
// the byte offsets of the centers' rows per tile and half plane.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void transpose_tables_kernel(const float* __restrict__ tables, int M,
                                                               float* __restrict__ tabT)
{
    // grid (256 subcodes c, M + 1): row (m, c) of the transposed tables; the row after the last table is +inf
    const int c = blockIdx.x, m = blockIdx.y, x = threadIdx.x;
    if (m == M) {
        if (c == 0) tabT[(size_t)M * L * L + x] = INFINITY;
        return;
    }
    tabT[((size_t)m * L + c) * L + x] = tables[((size_t)m * L + x) * L + c];
}

// rowoff[tile][2 m + h][kin] for M = 4, tiles of 32 centers: one thread per entry
__global__ __launch_bounds__(256) void tile_rows4_kernel(const uint8_t* __restrict__ centers, int K,
                                                         uint32_t* __restrict__ rowoff, int64_t total)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int kin = (int)(e & 15), pl = (int)((e >> 4) & 7);
    const int64_t tile = e >> 7;
    const int m = pl >> 1, h = pl & 1;
    const int64_t k = tile * 32 + 16 * h + kin;
    rowoff[e] = (k < K) ? (uint32_t)(m * L + centers[k * 4 + m]) * 1024u : (uint32_t)(4 * L) * 1024u;
}

// ---------------------------------------------------------------------------------------------
// M = 4 scan over residue-grouped codes with slots of TWO lanes (16 centers per lane).
//
// Same tile image, same arithmetic and same regrouping idea as assign_scan4p_kernel, but a code is worked on by
// two lanes instead of four, so a workgroup of 512 threads holds 256 R codes per tile fill instead of 128 R: the
// 128 KB fill, which the LDS takes at a quarter of its read rate, is shared by twice as many codes.  A lane
// reads, per subspace, two 16-byte pieces of each of the two half planes: the 32 bytes of its slot's half of the
// 64-byte plane row first, then (address ^ 32) the other half.  An LDS access serves eight slots; the four even
// ones are one residue group (four different subcodes mod 4 in every subspace) and start with the lower halves,
// the four odd ones are another and start with the upper halves: sixteen different 16-byte positions in every
// read.  Per code and lane the state is what the four-lane scan keeps (two registers of packed row offsets, the
// running minimum, the tile in which it last improved); the winner inside the tile is recovered in the epilogue.
// ---------------------------------------------------------------------------------------------
// Where the tiles come from when they are not read as ready-made images: the transposed tables
// tabT[m][c][x] = A^m[x][c] (one contiguous 1 KB row per center subcode, plus one last row of +inf) and, per tile and
// half plane, the byte offsets of the rows of its 16 centers, rowoff[tile][2 m + h][16] (the +inf row for centers
// past K).  The tables are small enough (M x 256 KB) to stay in every L2, so a tile costs no HBM traffic at all,
// where the images (K x M KB, fetched again by every workgroup that has drifted out of step with its neighbours)
// cost the scan its whole HBM traffic.
struct TileSource {
    const float* tabT = nullptr;
    const uint32_t* rowoff = nullptr;
    uint32_t tab_bytes = 0;
};

template <int R, int THREADS, int DEPTH, bool TABLES = false>
__global__ __launch_bounds__(THREADS) void assign_scan4q_kernel(int64_t N, const uint2* __restrict__ gco,
                                                                const float4* __restrict__ img,
                                                                const float4* __restrict__ rows, int ntiles,
                                                                int32_t* __restrict__ assign,
                                                                float* __restrict__ dist, RankOut ro,
                                                                TileSource ts = TileSource{})
{
    constexpr int LPS = 2, TK = 32;
    constexpr int SLOTS = THREADS / LPS;
    constexpr int C = SLOTS * R;
    constexpr int NF = TILE_F4 / THREADS;
    constexpr uint32_t HPLANE = 16384;      // bytes per (m, h) plane: 256 subcodes x 16 centers
    static_assert(TILE_F4 % THREADS == 0, "tile must divide evenly over the workgroup");
    static_assert(R * THREADS * 8 <= TILE_BYTES, "the per-lane records must fit the tile buffer");
    static_assert(R % 2 == 0, "the epilogue gives every lane R / 2 codes");

    __shared__ float4 tile[TILE_F4];
    const char* tb = reinterpret_cast<const char*>(tile);

    const int tid = threadIdx.x;
    const int q = tid & 1;
    const int c = tid >> 1;
    const uint32_t hq = ((uint32_t)(c & 1) << 5) | ((uint32_t)q << 4);    // the slot's first half of the row, the lane's piece
    const int64_t base = (int64_t)blockIdx.x * C;
    const uint32_t low15 = 0x7fffu;

    uint32_t pa[R], pb[R];
    float best[R];
    int tix[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t n = base + (int64_t)r * SLOTS + c;
        if (n >= N) n = N - 1;
        const uint32_t pk = gco[n].x;
        const uint32_t f0 = ((pk & 255u) << 6) | hq;
        const uint32_t f1 = (((pk >> 8) & 255u) << 6) | hq;
        const uint32_t f2 = ((((pk >> 16) & 255u) << 6) | hq) + 65536u;
        const uint32_t f3 = (((pk >> 24) << 6) | hq) + 65536u;
        pa[r] = f0 | (f2 << 15);
        pb[r] = f1 | (f3 << 15);
        best[r] = INFINITY;
        tix[r] = -1;
    }

    const uint32_t lane_off = (uint32_t)tid * 16u;
    v4f* ltile = reinterpret_cast<v4f*>(tile);
    auto gload = [&](int t, int i) -> v4f {
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float4*>(img + (size_t)t * TILE_F4), 0, TILE_BYTES, 0x00020000);
        return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, i * THREADS * 16, 0));
    };
    // TABLES: float4 i*THREADS + tid of the tile is plane i/2, subcode x = (i&1)*128 + tid/4, piece p = tid&3: its four
    // entries are A^m[x][c] of the centers 16h + 4p + j, i.e. element x of four rows of the transposed tables
    const uint32_t x4 = (uint32_t)(tid >> 2) * 4u;
    const uint32_t ro_lane = (uint32_t)(tid & 3) * 16u;
    auto ro_load = [&](int t, int pl) -> uint4 {
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint32_t*>(ts.rowoff + (size_t)t * 128), 0, 512, 0x00020000);
        return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs, ro_lane, pl * 64, 0));
    };
    __amdgpu_buffer_rsrc_t rs_tab = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(ts.tabT), 0, ts.tab_bytes,
                                                                      0x00020000);
    v4f pf[NF];
    auto plane_load = [&](const uint4 rof, int pl) {
        const uint32_t o0 = rof.x + x4, o1 = rof.y + x4, o2 = rof.z + x4, o3 = rof.w + x4;
        pf[2 * pl].x = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_tab, o0, 0, 0));
        pf[2 * pl].y = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_tab, o1, 0, 0));
        pf[2 * pl].z = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_tab, o2, 0, 0));
        pf[2 * pl].w = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_tab, o3, 0, 0));
        pf[2 * pl + 1].x = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_tab, o0, 512, 0));
        pf[2 * pl + 1].y = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_tab, o1, 512, 0));
        pf[2 * pl + 1].z = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_tab, o2, 512, 0));
        pf[2 * pl + 1].w = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_tab, o3, 512, 0));
    };
    uint4 rnext = make_uint4(0u, 0u, 0u, 0u);      // row offsets of the plane whose loads are issued next
    if (TABLES) {
        static_assert(!TABLES || (THREADS == 512 && NF == 16), "the table-built tile assumes 512 threads");
        rnext = ro_load(0, 0);
#pragma unroll
        for (int pl = 0; pl < 8; ++pl) {
            const uint4 cur = rnext;
            rnext = pl < 7 ? ro_load(0, pl + 1) : ro_load(ntiles > 1 ? 1 : 0, 0);
            plane_load(cur, pl);
        }
    } else {
#pragma unroll
        for (int i = 0; i < NF; ++i) pf[i] = gload(0, i);
    }

    // a step is one subspace of one code: four 16-byte reads (two pieces of each half plane)
    struct Quad { float4 a, b, c, d; };
    auto issue = [&](int step) -> Quad {
        const int r = step / 4, m = step % 4;
        const uint32_t ad = (m == 0) ? unpack_low15(low15, pa[r])
                          : (m == 1) ? unpack_low15(low15, pb[r])
                          : (m == 2) ? unpack_high17(pa[r])
                                     : unpack_high17(pb[r]);
        const uint32_t ad2 = ad ^ 32u;
        const uint32_t po = (m & 1) ? 2 * HPLANE : 0;
        Quad p;
        p.a = lds_read16(tb, ad + po);
        p.b = lds_read16(tb, ad2 + po);
        p.c = lds_read16(tb, ad + po + HPLANE);
        p.d = lds_read16(tb, ad2 + po + HPLANE);
        return p;
    };

    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NF; ++i) ltile[i * THREADS + tid] = pf[i];
        __syncthreads();
        const int tn = t + 1 < ntiles ? t + 1 : t;
        Quad ring[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) ring[d] = issue(d);
        float4 sa, sb, sc, sd;
        const int tnn = tn + 1 < ntiles ? tn + 1 : tn;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (TABLES) {
                // the eight planes of the next tile, spread over the first 5/8 of the scan; with each the row
                // offsets of the plane after it (those of plane 0 of the tile after next come with plane 7)
#pragma unroll
                for (int pl = 0; pl < 8; ++pl)
                    if ((2 * pl * R * 5) / (NF * 8) == r) {
                        const uint4 cur = rnext;
                        rnext = pl < 7 ? ro_load(tn, pl + 1) : ro_load(tnn, 0);
                        plane_load(cur, pl);
                    }
            } else {
#pragma unroll
                for (int i = 0; i < NF; ++i)
                    if ((i * R * 5) / (NF * 8) == r) pf[i] = gload(tn, i);
            }
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const int step = 4 * r + m;
                const Quad cur = ring[step % DEPTH];
                if (step + DEPTH < 4 * R) ring[step % DEPTH] = issue(step + DEPTH);
                if (m == 0) {
                    sa = cur.a; sb = cur.b; sc = cur.c; sd = cur.d;
                } else {
                    sa.x = sa.x + cur.a.x; sa.y = sa.y + cur.a.y; sa.z = sa.z + cur.a.z; sa.w = sa.w + cur.a.w;
                    sb.x = sb.x + cur.b.x; sb.y = sb.y + cur.b.y; sb.z = sb.z + cur.b.z; sb.w = sb.w + cur.b.w;
                    sc.x = sc.x + cur.c.x; sc.y = sc.y + cur.c.y; sc.z = sc.z + cur.c.z; sc.w = sc.w + cur.c.w;
                    sd.x = sd.x + cur.d.x; sd.y = sd.y + cur.d.y; sd.z = sd.z + cur.d.z; sd.w = sd.w + cur.d.w;
                }
                if (m == 3) {
                    float m16 = min3_f32(sa.x, sa.y, sa.z);
                    m16 = min3_f32(m16, sa.w, sb.x);
                    m16 = min3_f32(m16, sb.y, sb.z);
                    m16 = min3_f32(m16, sb.w, sc.x);
                    m16 = min3_f32(m16, sc.y, sc.z);
                    m16 = min3_f32(m16, sc.w, sd.x);
                    m16 = min3_f32(m16, sd.y, sd.z);
                    const float nb = min3_f32(m16, sd.w, best[r]);
                    tix[r] = (nb < best[r]) ? t : tix[r];
                    best[r] = nb;
                }
            }
        }
    }

    // Epilogue, transposed through LDS as in assign_scan4p_kernel: every lane leaves (minimum, tile) per code, then
    // lane l finishes the codes l, l + THREADS, ...: the slot minimum is the smaller of the two lanes' minima, the
    // winning tile the lowest tile among the lanes that attain it, and for every lane position that attains it in
    // that tile the 16 sums of its centers are rebuilt from the row-ordered copy of the images ([tile][m][x][32
    // centers]: same bits, same order of additions) and the lowest center index with that sum is kept.
    constexpr int CPL = R / 2;
    __syncthreads();
    {
        float2* rec = reinterpret_cast<float2*>(tile);
#pragma unroll
        for (int r = 0; r < R; ++r)                  // record index = 2 * (code index in the workgroup) + q
            rec[(r * SLOTS + c) * 2 + q] = make_float2(best[r], __builtin_bit_cast(float, tix[r]));
    }
    __syncthreads();
    __amdgpu_buffer_rsrc_t rs_img = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float4*>(rows), 0, (uint32_t)ntiles * (uint32_t)TILE_BYTES, 0x00020000);
    constexpr int TNONE = 0x7fffffff;
#pragma unroll 1
    for (int i0 = 0; i0 < CPL; ++i0) {
        const int jj = i0 * THREADS + tid;           // code index in the workgroup: slot jj % SLOTS, round jj / SLOTS
        int64_t n = base + jj;
        const bool live = n < N;
        if (!live) n = N - 1;
        const float4 ra = lds_read16(tb, (uint32_t)jj * 16u);
        const float b0 = ra.x, b1 = ra.z;
        const int t0 = __builtin_bit_cast(int, ra.y), t1 = __builtin_bit_cast(int, ra.w);
        const float sm = __builtin_fminf(b0, b1);
        const int c0 = (b0 == sm && t0 >= 0) ? t0 : TNONE, c1 = (b1 == sm && t1 >= 0) ? t1 : TNONE;
        const int tm = c0 < c1 ? c0 : c1;
        uint32_t cand = (uint32_t)(c0 == tm) | ((uint32_t)(c1 == tm) << 1);
        if (tm == TNONE || !live) cand = 0u;
        const uint2 g = gco[n];
        const uint32_t pk = g.x;
        const uint32_t og = live ? g.y : ORIGIN_NONE;
        const uint32_t hs = (uint32_t)((jj % SLOTS) & 1);      // which half of the row the code's slot read first
        int bi = IDX_NONE;
        while (__any(cand != 0u)) {                  // one trip unless the two lane positions tie exactly
            const uint32_t qe = cand ? (uint32_t)__builtin_ctz(cand) : 0u;
            // lane position qe of a slot with first half hs owns the pieces p = 2 hs' + qe of both halves of the row:
            // first read hs' = hs (centers 4 p .. 4 p + 3 and 16 + 4 p ..), second read hs' = 1 - hs
            const uint32_t pA = 2u * hs + qe, pB = 2u * (1u - hs) + qe;
            const uint32_t tb0 = cand ? (uint32_t)tm * (uint32_t)TILE_BYTES : 0xfff00000u;
            v4f sA, sB, sC, sD;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const uint32_t x = (pk >> (8 * m)) & 255u;
                const uint32_t o = tb0 + (x << 7);
                constexpr int MP = 32768;             // bytes per subspace in a tile of the row copy
                const v4f vA = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o + pA * 16u, m * MP, 0));
                const v4f vB = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o + pB * 16u, m * MP, 0));
                const v4f vC = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o + pA * 16u, m * MP + 64, 0));
                const v4f vD = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o + pB * 16u, m * MP + 64, 0));
                if (m == 0) { sA = vA; sB = vB; sC = vC; sD = vD; }
                else { sA = sA + vA; sB = sB + vB; sC = sC + vC; sD = sD + vD; }
            }
            if (cand) {
                const int kt = tm * TK;
                const int kA = kt + (int)pA * 4, kB = kt + (int)pB * 4, kC = kA + 16, kD = kB + 16;
                int k = IDX_NONE;
                auto take = [&](const v4f& v, int k0) {
                    int kk = IDX_NONE;
                    if (v.w == sm) kk = k0 + 3;
                    if (v.z == sm) kk = k0 + 2;
                    if (v.y == sm) kk = k0 + 1;
                    if (v.x == sm) kk = k0;
                    k = kk < k ? kk : k;
                };
                take(sA, kA); take(sB, kB); take(sC, kC); take(sD, kD);
                bi = k < bi ? k : bi;
                cand &= cand - 1u;
            }
        }
        if (og != ORIGIN_NONE) {
            const int kw = (bi == IDX_NONE) ? 0 : bi;
            assign[og] = kw;
            if (dist) dist[og] = sm;
            if (ro.count) ro.rank[og] = atomicAdd(&ro.count[kw], 1u);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// M = 4 scan with two-lane slots whose tiles arrive in LDS without passing through registers.
//
// Same regrouped codes, same tile image (img[tile][m][h][x][16 centers]), same packed offsets and the same sums as
// assign_scan4q_kernel.  What differs is how a tile gets into LDS.  There the next tile waits in 64 registers per
// lane and is written between two barriers, while no wave can read; here the two halves of a tile (h = 0: its
// first 16 centers, h = 1: the other 16; 64 KB each, the planes [m][h] of both interleaved exactly as in the image)
// are two buffers: while the workgroup scans one half, buffer loads with the LDS as their destination bring the
// half after it into the other one, 16 bytes per lane and 1 KB per wave and instruction, and a wave waits for its
// own loads only at the one barrier per half.  The registers that held the prefetch hold more codes instead (a
// 64 KB fill is shared by 256 R codes with R up to 48), and the LDS never idles for a fill.  The price: a code
// passes over its tile twice (once per half), so a step is two 16-byte reads instead of four for the same unpack
// and xor.  Per code and lane: two registers of packed row offsets, the running minimum, the HALF tile
// (2 tile + h) in which it last improved.
// ---------------------------------------------------------------------------------------------
typedef int v4i __attribute__((ext_vector_type(4)));

// 16 bytes per lane from a buffer straight into LDS: lane l of the wave writes LDS bytes lds_addr + 16 l .. + 15
// (lds_addr is the same for the whole wave) with the 16 bytes at buffer offset voffset + soffset.  Counted like
// any other vector memory load (s_waitcnt vmcnt).
__device__ __forceinline__ void buffer_to_lds16(uint32_t lds_addr, v4i rsrc, uint32_t voffset, uint32_t soffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
                 : "memory", "m0");
}
__device__ __forceinline__ void wait_vector_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int R, int THREADS, int DEPTH, bool BUCKET = false>
__global__ __launch_bounds__(THREADS) void assign_scan4h_kernel(int64_t N, const uint2* __restrict__ gco,
                                                            const float4* __restrict__ img,
                                                            const float4* __restrict__ rows, int ntiles, int nhalves,
                                                            int32_t* __restrict__ assign, float* __restrict__ dist,
                                                            RankOut ro, BucketOut bo = BucketOut{})
{
    constexpr int LPS = 2, TK = 32;
    constexpr int SLOTS = THREADS / LPS;
    constexpr int C = SLOTS * R;
    constexpr uint32_t HPLANE = 16384;      // bytes per (m, h) plane: 256 subcodes x 16 centers
    static_assert(R % 2 == 0, "the epilogue gives every lane R / 2 codes");
    static_assert(C * 8 <= TILE_BYTES, "one 8-byte record per code must fit the tile buffer");
    static_assert(!BUCKET || C * 24 <= TILE_BYTES, "BUCKET: 16 more bytes per code behind the records");
    // BUCKET: the workgroup also files its codes by cluster group for the histogram, as assign_scan4p_kernel does
    // (the whole grid must be one launch: segment (g, w) is named by blockIdx.x and gridDim.x)
    __shared__ uint32_t gcnt[BUCKET ? 256 : 1];
    __shared__ uint32_t gbase[BUCKET ? 256 : 1];

    __shared__ float4 tile[TILE_F4];
    const char* tb = reinterpret_cast<const char*>(tile);

    const int tid = threadIdx.x;
    const int q = tid & 1;
    const int c = tid >> 1;
    const uint32_t hq = ((uint32_t)(c & 1) << 5) | ((uint32_t)q << 4);    // the slot's first half of the row, the lane's piece
    const int64_t base = (int64_t)blockIdx.x * C;
    const uint32_t low15 = 0x7fffu;

    // the whole image as one buffer; the workgroup brings in a half (t, h) in NCH chunks of 16 bytes per lane
    constexpr uint32_t CHUNK = THREADS * 16;
    constexpr int NCH = 4 * HPLANE / CHUNK;
    static_assert(HPLANE % CHUNK == 0 || CHUNK % HPLANE == 0, "a chunk is a whole plane or a whole fraction of one");
    const uint64_t ip = reinterpret_cast<uint64_t>(img);
    const v4i rs_img = {(int)(uint32_t)ip, (int)(uint32_t)(ip >> 32), (int)((uint32_t)ntiles * (uint32_t)TILE_BYTES),
                        0x00020000};
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)tile;    // LDS byte address of the buffer
    const uint32_t wave_off = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6) * 1024u;
    const uint32_t lane_off = (uint32_t)tid * 16u;
    auto fetch = [&](int t, int h, int j) {
        const uint32_t in_half = (uint32_t)j * CHUNK;                // plane m = in_half / HPLANE of the half
        const uint32_t in_tile = (in_half / HPLANE) * (2 * HPLANE) + (uint32_t)h * HPLANE + in_half % HPLANE;
        buffer_to_lds16(lds0 + in_tile + wave_off, rs_img, lane_off, (uint32_t)t * (uint32_t)TILE_BYTES + in_tile);
    };
#pragma unroll
    for (int j = 0; j < NCH; ++j) fetch(0, 0, j);

    uint32_t pa[R], pb[R];
    float best[R];
    int tix[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t n = base + (int64_t)r * SLOTS + c;
        if (n >= N) n = N - 1;
        const uint32_t pk = gco[n].x;
        const uint32_t f0 = ((pk & 255u) << 6) | hq;
        const uint32_t f1 = (((pk >> 8) & 255u) << 6) | hq;
        const uint32_t f2 = ((((pk >> 16) & 255u) << 6) | hq) + 65536u;
        const uint32_t f3 = (((pk >> 24) << 6) | hq) + 65536u;
        pa[r] = f0 | (f2 << 15);
        pb[r] = f1 | (f3 << 15);
        best[r] = INFINITY;
        tix[r] = -1;
    }

    // a step is one subspace of one code in one half: two 16-byte reads (the lane's piece of either half of the row)
    struct Pair { float4 a, b; };

    for (int t = 0; t < ntiles; ++t) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            // this half has arrived (own loads, then everybody's), and nobody reads the other buffer any more
            // (nhalves = the halves that hold a center, 2 ntiles or one less: an all-padding last half is not scanned)
            if (2 * t + h >= nhalves) break;
            wait_vector_loads();
            __syncthreads();
            const int tf = h ? t + 1 : t, hf = h ^ 1;                // the half after this one
            const bool more = 2 * t + h + 1 < nhalves;
            auto issue = [&](int step) -> Pair {
                const int r = step / 4, m = step % 4;
                const uint32_t ad = (m == 0) ? unpack_low15(low15, pa[r])
                                  : (m == 1) ? unpack_low15(low15, pb[r])
                                  : (m == 2) ? unpack_high17(pa[r])
                                             : unpack_high17(pb[r]);
                const uint32_t po = ((m & 1) ? 2 * HPLANE : 0) + h * HPLANE;
                Pair p;
                p.a = lds_read16(tb, ad + po);
                p.b = lds_read16(tb, (ad ^ 32u) + po);
                return p;
            };
            Pair ring[DEPTH];
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) ring[d] = issue(d);
            float4 sa, sb;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                // the chunks of the next half, spread over the first half of the codes
#pragma unroll
                for (int j = 0; j < NCH; ++j)
                    if ((j * R) / (2 * NCH) == r && more) fetch(tf, hf, j);
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const int step = 4 * r + m;
                    const Pair cur = ring[step % DEPTH];
                    if (step + DEPTH < 4 * R) ring[step % DEPTH] = issue(step + DEPTH);
                    if (m == 0) {
                        sa = cur.a; sb = cur.b;
                    } else {
                        sa.x = sa.x + cur.a.x; sa.y = sa.y + cur.a.y; sa.z = sa.z + cur.a.z; sa.w = sa.w + cur.a.w;
                        sb.x = sb.x + cur.b.x; sb.y = sb.y + cur.b.y; sb.z = sb.z + cur.b.z; sb.w = sb.w + cur.b.w;
                    }
                    if (m == 3) {
                        float m8 = min3_f32(sa.x, sa.y, sa.z);
                        m8 = min3_f32(m8, sa.w, sb.x);
                        m8 = min3_f32(m8, sb.y, sb.z);
                        const float nb = min3_f32(m8, sb.w, best[r]);
                        tix[r] = (nb < best[r]) ? 2 * t + h : tix[r];
                        best[r] = nb;
                    }
                }
            }
        }
    }

    // Epilogue.  The two lanes of a slot merge what they hold (the neighbour's minimum and half tile through a lane
    // permutation): slot minimum, the lowest half tile among the lanes that attain it, and which lane positions do so
    // there; one of them leaves that as the code's 8-byte record in LDS.  Then lane l finishes the codes l, l + THREADS,
    // ...: for every lane position named by the record the 8 sums of its centers in that half are rebuilt from the
    // row-ordered copy of the images ([tile][m][x][32 centers]: same bits, same order of additions) and the lowest
    // center index with that sum is kept.
    constexpr int CPL = R / 2;
    constexpr int TNONE = 0x7fffffff;
    if (BUCKET && tid < 256) gcnt[tid] = 0u;
    __syncthreads();
    {
        uint2* rec = reinterpret_cast<uint2*>(tile);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float ob = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, best[r]), 0xB1, 0xf, 0xf, true));
            const int ot = __builtin_amdgcn_update_dpp(0, tix[r], 0xB1, 0xf, 0xf, true);      // lanes 2 i and 2 i + 1 swapped
            const float sm = __builtin_fminf(best[r], ob);
            const int cm = (best[r] == sm && tix[r] >= 0) ? tix[r] : TNONE, co = (ob == sm && ot >= 0) ? ot : TNONE;
            const int um = cm < co ? cm : co;
            const uint32_t mine = (uint32_t)(cm == um), other = (uint32_t)(co == um);
            const uint32_t cand = (um == TNONE) ? 0u : (q ? (other | (mine << 1)) : (mine | (other << 1)));
            if (q == (r & 1))
                rec[r * SLOTS + c] = make_uint2(__builtin_bit_cast(uint32_t, sm), (um == TNONE ? 0u : (uint32_t)um) | (cand << 30));
        }
    }
    __syncthreads();
    __amdgpu_buffer_rsrc_t rs_rows = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float4*>(rows), 0, (uint32_t)ntiles * (uint32_t)TILE_BYTES, 0x00020000);
#pragma unroll 1
    for (int i0 = 0; i0 < CPL; ++i0) {
        const int jj = i0 * THREADS + tid;           // code index in the workgroup: slot jj % SLOTS, round jj / SLOTS
        int64_t n = base + jj;
        const bool live = n < N;
        if (!live) n = N - 1;
        const uint2 rc = reinterpret_cast<const uint2*>(tile)[jj];
        const float sm = __builtin_bit_cast(float, rc.x);
        const int um = (int)(rc.y & 0x3fffffffu);
        uint32_t cand = live ? (rc.y >> 30) : 0u;
        const int tm = um >> 1;
        const uint32_t h = (uint32_t)(um & 1);
        const uint2 g = gco[n];
        const uint32_t pk = g.x;
        const uint32_t og = live ? g.y : ORIGIN_NONE;
        const uint32_t hs = (uint32_t)(jj & 1);      // which half of the row the code's slot read first
        int bi = IDX_NONE;
        while (__any(cand != 0u)) {                  // one trip unless the two lane positions tie exactly
            const uint32_t qe = cand ? (uint32_t)__builtin_ctz(cand) : 0u;
            // lane position qe of a slot with first half hs owns the pieces 2 hs + qe (first read) and 2 (1 - hs) + qe
            const uint32_t pA = 2u * hs + qe, pB = 2u * (1u - hs) + qe;
            const uint32_t tb0 = cand ? (uint32_t)tm * (uint32_t)TILE_BYTES + h * 64u : 0xfff00000u;
            v4f sA, sB;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const uint32_t x = (pk >> (8 * m)) & 255u;
                const uint32_t o = tb0 + (x << 7);
                constexpr int MP = 32768;             // bytes per subspace in a tile of the row copy
                const v4f vA = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_rows, o + pA * 16u, m * MP, 0));
                const v4f vB = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_rows, o + pB * 16u, m * MP, 0));
                if (m == 0) { sA = vA; sB = vB; }
                else { sA = sA + vA; sB = sB + vB; }
            }
            if (cand) {
                const int kt = tm * TK + 16 * (int)h;
                const int kA = kt + (int)pA * 4, kB = kt + (int)pB * 4;
                int k = IDX_NONE;
                auto take = [&](const v4f& v, int k0) {
                    int kk = IDX_NONE;
                    if (v.w == sm) kk = k0 + 3;
                    if (v.z == sm) kk = k0 + 2;
                    if (v.y == sm) kk = k0 + 1;
                    if (v.x == sm) kk = k0;
                    k = kk < k ? kk : k;
                };
                take(sA, kA); take(sB, kB);
                bi = k < bi ? k : bi;
                cand &= cand - 1u;
            }
        }
        if (og != ORIGIN_NONE) {
            const int kw = (bi == IDX_NONE) ? 0 : bi;
            assign[og] = kw;
            if (dist) dist[og] = sm;
            if (ro.count) ro.rank[og] = atomicAdd(&ro.count[kw], 1u);
        }
        if (BUCKET) {
            // behind the 8-byte records: the code, its center, its cluster group and its rank among the workgroup's
            // codes of that group
            const uint32_t k = (bi == IDX_NONE) ? 0u : (uint32_t)bi;
            uint32_t g = 0xffffffffu, rank = 0u;
            if (og != ORIGIN_NONE) {
                g = k / (uint32_t)bo.KT;
                g = g < 255u ? g : 255u;                         // k < K and at most 255 groups: never taken
                rank = atomicAdd(&gcnt[g], 1u);
            }
            *reinterpret_cast<uint4*>(reinterpret_cast<char*>(tile) + (size_t)C * 8 + (size_t)jj * 16u) = make_uint4(pk, k, g, rank);
        }
    }
    if (BUCKET) {
        __syncthreads();
        if (tid < 64) {                                          // exclusive prefix over the groups: lane l owns 4l .. 4l+3
            const uint32_t a0 = gcnt[4 * tid], a1 = gcnt[4 * tid + 1], a2 = gcnt[4 * tid + 2], a3 = gcnt[4 * tid + 3];
            const uint32_t mine = a0 + a1 + a2 + a3;
            const uint32_t e0 = wave_inclusive_scan(mine) - mine, e1 = e0 + a0, e2 = e1 + a1, e3 = e2 + a2;
            gbase[4 * tid] = e0;  gbase[4 * tid + 1] = e1;  gbase[4 * tid + 2] = e2;  gbase[4 * tid + 3] = e3;
            const size_t nw = gridDim.x;
            uint2* sg = bo.seg + blockIdx.x;
            if (4 * tid < bo.ngroups) sg[(size_t)(4 * tid) * nw] = make_uint2((uint32_t)(base + e0), a0);
            if (4 * tid + 1 < bo.ngroups) sg[(size_t)(4 * tid + 1) * nw] = make_uint2((uint32_t)(base + e1), a1);
            if (4 * tid + 2 < bo.ngroups) sg[(size_t)(4 * tid + 2) * nw] = make_uint2((uint32_t)(base + e2), a2);
            if (4 * tid + 3 < bo.ngroups) sg[(size_t)(4 * tid + 3) * nw] = make_uint2((uint32_t)(base + e3), a3);
        }
        __syncthreads();
#pragma unroll 1
        for (int i = 0; i < CPL; ++i) {
            const int j = i * THREADS + tid;
            const uint4 r = *reinterpret_cast<const uint4*>(tb + (size_t)C * 8 + (size_t)j * 16u);
            if (r.z != 0xffffffffu) bo.pool[base + gbase[r.z] + r.w] = make_uint2(r.x, r.y);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Eq. 7 from the records the scan filed by cluster group (M = 4): workgroup (g, s) owns group g
// (KT clusters, private histograms in LDS as in the owner path) and the scan workgroups
// w = s, s + S, ...; each of its waves takes some of them, reads group g's stretch of their
// records (contiguous, (code, center) pairs) and counts with LDS atomics.  No pass over the
// assignment array, no gather of codes: 8 bytes per code are read once.  Output as the owner
// path's: the private histograms whole, S partial arrays when S > 1.
// ---------------------------------------------------------------------------------------------
template <int LDS_WORDS>
__global__ __launch_bounds__(1024) void histogram_bucket_kernel(const uint2* __restrict__ pool,
                                                                const uint2* __restrict__ seg, int nwg, int K,
                                                                int KT, int S, uint32_t* __restrict__ hist,
                                                                size_t part_stride)
{
    constexpr int M = 4;
    __shared__ uint32_t lh[LDS_WORDS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x / S, s = blockIdx.x % S;
    const int k0 = g * KT;
    const int kt = (K - k0 < KT) ? K - k0 : KT;
    const int words = kt * M * L;
    for (int i = tid; i < words; i += 1024) lh[i] = 0u;
    __syncthreads();
    constexpr int SB = 4;                                   // segments whose records are in flight together
    const int stride = 16 * S;
    for (int w0 = s * 16 + wave; w0 < nwg; w0 += stride * SB) {
        uint2 sg[SB];
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            const int w = w0 + u * stride;
            sg[u] = w < nwg ? seg[(size_t)g * nwg + w] : make_uint2(0u, 0u);
        }
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            for (uint32_t i = lane; i < sg[u].y; i += 64) {
                const uint2 r = pool[(size_t)sg[u].x + i];
                const uint32_t kk = r.y - (uint32_t)k0;
                if (kk < (uint32_t)kt) {
                    uint32_t* h = lh + (size_t)kk * M * L;
                    atomicAdd(&h[0 * L + (r.x & 255u)], 1u);
                    atomicAdd(&h[1 * L + ((r.x >> 8) & 255u)], 1u);
                    atomicAdd(&h[2 * L + ((r.x >> 16) & 255u)], 1u);
                    atomicAdd(&h[3 * L + (r.x >> 24)], 1u);
                }
            }
        }
    }
    __syncthreads();
    uint32_t* out = hist + (size_t)s * part_stride + (size_t)k0 * M * L;
    for (int i = tid; i < words; i += 1024) out[i] = lh[i];
}

// ---------------------------------------------------------------------------------------------
// M = 8 (64-bit codes): regrouping and scan with conflict-free reads, as for M = 4.
//
// A tile is 16 centers, img[tile][m][x][16]: plane m at byte m*16384, row x of 64 bytes, so the
// bank quarter of a slot's read is x mod 4 in each of its 8 reads.  A group of four codes reads
// conflict-free when their subcodes differ mod 4 in all eight subspaces; the class of a code is
// now 16 bits (65536 classes), the orbits are again c, c^a, c^b, c^a^b for masks whose 2-bit fields
// are non-zero and different in every subspace, and the plan is the same greedy matching over a
// fixed list of mask pairs.  With 65536 classes the per-class counters live in global memory:
// ranks come from one global atomic per code (spread over 65536 addresses), so the order inside
// a class is not fixed from run to run -- the results are, since the scan treats every code alone.
// The scan needs no skew steps: 8 reads and 28 adds per 4 evaluations where the skewed scan below
// has 11 and 40.
// ---------------------------------------------------------------------------------------------
constexpr int GROUP8_CLASSES = 65536;
constexpr int GROUP8_ORBITS = GROUP8_CLASSES / 4;

__constant__ uint16_t group8_masks[GROUP_ROUNDS][2] = {
    {0x6b55, 0xd6ee}, {0x76e5, 0xd99f}, {0xb7eb, 0x5a96}, {0xfa6e, 0xa5b7}, {0x6b66, 0xdefd}, {0xe76b, 0xbad6},
    {0x5ebb, 0xb9ee}, {0xa69a, 0x7d67}, {0x6afe, 0xdfab}, {0x799d, 0x9ffa}, {0x97f7, 0x6e69}, {0x9d7d, 0xf6eb},
    {0xbf66, 0xe9f9}, {0xd5ad, 0xbbfb}, {0xdd95, 0xa6fa}, {0x9f59, 0x69ff}};

struct GroupPlan8 {
    uint32_t count[GROUP8_CLASSES];                       // codes per class
    uint32_t cursor[GROUP8_CLASSES];                      // codes handed out so far (scatter pass)
    uint32_t rem[GROUP_ROUNDS + 1][GROUP8_CLASSES];       // [d][class]: codes of the class not matched before round d; [last] = left over
    uint32_t gbase[GROUP_ROUNDS][GROUP8_CLASSES];         // [d][class]: index of the first group the class's orbit forms in round d
    uint32_t lbase[GROUP8_CLASSES];                       // index of the class's first left-over code among all left-overs
    uint32_t groups, leftovers, lgroups, period_m1;
};

__device__ __forceinline__ uint32_t code8_class(uint32_t lo, uint32_t hi)
{
    return code_class(lo) | (code_class(hi) << 8);
}

__global__ __launch_bounds__(256) void code8_class_count_kernel(const uint8_t* __restrict__ codes, int64_t n,
                                                                GroupPlan8* __restrict__ plan)
{
    const uint2* cw = reinterpret_cast<const uint2*>(codes);
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (; i < n; i += stride) {
        const uint2 v = cw[i];
        atomicAdd(&plan->count[code8_class(v.x, v.y)], 1u);
    }
}

// one workgroup of 1024 threads: thread t owns the orbits t, t + 1024, ... of every round (an orbit is named by its
// class with residue 0 in subspace 0, class = 4 * orbit index; groups are numbered in orbit order).  The tables
// are stored round-major so that the 64 lanes of a wave touch one kilobyte per access.
__global__ __launch_bounds__(1024) void code8_group_plan_kernel(GroupPlan8* __restrict__ plan)
{
    constexpr int OPT = GROUP8_ORBITS / 1024;      // orbits per thread
    __shared__ uint32_t wsum[OPT][16];             // per stripe of 1024 orbits and wave: groups formed
    __shared__ uint32_t sbase[OPT];                // per stripe: groups formed by the stripes before it
    __shared__ uint32_t round_total;
    const int tid = threadIdx.x, wv = tid >> 6;
    for (int c = tid; c < GROUP8_CLASSES; c += 1024) {
        plan->rem[0][c] = plan->count[c];
        plan->cursor[c] = 0u;
    }
    __syncthreads();
    uint32_t gtot = 0;
    for (int d = 0; d < GROUP_ROUNDS; ++d) {
        const uint32_t a = group8_masks[d][0], b = group8_masks[d][1];
        uint32_t m[OPT], r0[OPT], r1[OPT], r2[OPT], r3[OPT], inc[OPT];
#pragma unroll
        for (int i = 0; i < OPT; ++i) {
            const uint32_t c0 = (uint32_t)(i * 1024 + tid) << 2;
            // values written by other threads of this workgroup in the previous round: read past the L1
            r0[i] = __hip_atomic_load(&plan->rem[d][c0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r1[i] = __hip_atomic_load(&plan->rem[d][c0 ^ a], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r2[i] = __hip_atomic_load(&plan->rem[d][c0 ^ b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r3[i] = __hip_atomic_load(&plan->rem[d][c0 ^ a ^ b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int i = 0; i < OPT; ++i) {
            uint32_t v = r0[i] < r1[i] ? r0[i] : r1[i];
            v = v < r2[i] ? v : r2[i];
            v = v < r3[i] ? v : r3[i];
            m[i] = v;
            inc[i] = wave_inclusive_scan(v);
            if ((tid & 63) == 63) wsum[i][wv] = inc[i];
        }
        __syncthreads();
        if (tid < OPT) {
            // exclusive prefix of the stripe totals: thread i sums the stripes before stripe i
            uint32_t e = 0;
            for (int ii = 0; ii < tid; ++ii)
                for (int w = 0; w < 16; ++w) e += wsum[ii][w];
            sbase[tid] = e;
            if (tid == OPT - 1) {
                uint32_t t = e;
                for (int w = 0; w < 16; ++w) t += wsum[OPT - 1][w];
                round_total = t;
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < OPT; ++i) {
            uint32_t before = gtot + sbase[i] + inc[i] - m[i];
            for (int w = 0; w < wv; ++w) before += wsum[i][w];
            const uint32_t c0 = (uint32_t)(i * 1024 + tid) << 2, c1 = c0 ^ a, c2 = c0 ^ b, c3 = c0 ^ a ^ b;
            plan->gbase[d][c0] = before;
            plan->gbase[d][c1] = before;
            plan->gbase[d][c2] = before;
            plan->gbase[d][c3] = before;
            plan->rem[d + 1][c0] = r0[i] - m[i];
            plan->rem[d + 1][c1] = r1[i] - m[i];
            plan->rem[d + 1][c2] = r2[i] - m[i];
            plan->rem[d + 1][c3] = r3[i] - m[i];
        }
        gtot += round_total;
        __syncthreads();               // rem[d+1] complete; wsum, sbase, round_total free for the next round
    }
    // left-overs: exclusive prefix over the classes in the order of leftover_order_class, thread t owns places
    // 64t .. 64t+63 of it
    {
        constexpr int CPT = GROUP8_CLASSES / 1024;
        uint32_t mine = 0;
        for (int i = 0; i < CPT; ++i)
            mine += __hip_atomic_load(&plan->rem[GROUP_ROUNDS][leftover_order_class((uint32_t)(tid * CPT + i), 8)],
                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t inc = wave_inclusive_scan(mine);
        if ((tid & 63) == 63) wsum[0][wv] = inc;
        __syncthreads();
        uint32_t e = inc - mine;
        for (int w = 0; w < wv; ++w) e += wsum[0][w];
        for (int i = 0; i < CPT; ++i) {
            const uint32_t cls = leftover_order_class((uint32_t)(tid * CPT + i), 8);
            plan->lbase[cls] = e;
            e += __hip_atomic_load(&plan->rem[GROUP_ROUNDS][cls], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (tid == 1023) {
            const uint32_t ltot = e, lg = (ltot + 3u) / 4u;
            plan->groups = gtot;
            plan->leftovers = ltot;
            plan->lgroups = lg;
            plan->period_m1 = (lg > 0 && gtot >= lg) ? gtot / lg : 0u;
        }
    }
}

// gc8[pos] = (code low word, code high word, original index, 0); positions that receive no code get ORIGIN_NONE
__global__ __launch_bounds__(256) void code8_group_scatter_kernel(const uint8_t* __restrict__ codes, int64_t n,
                                                                  GroupPlan8* __restrict__ plan,
                                                                  uint4* __restrict__ gc8, int64_t n_alloc,
                                                                  int blocks_of_16 = 0)
{
    const uint2* cw = reinterpret_cast<const uint2*>(codes);
    const uint32_t gtot = plan->groups, ltot = plan->leftovers, lg = plan->lgroups, dm1 = plan->period_m1;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (; i < n; i += stride) {
        const uint2 v = cw[i];
        const uint32_t c = code8_class(v.x, v.y);
        const uint32_t rank = atomicAdd(&plan->cursor[c], 1u);
        const uint32_t tot = plan->rem[0][c];
        const uint32_t left = plan->rem[GROUP_ROUNDS][c];
        int64_t u;
        uint32_t slot;
        if (rank < tot - left) {
            // round d took the ranks [tot - rem[d], tot - rem[d+1]): largest d with tot - rem[d] <= rank
            int d = 0;
#pragma unroll
            for (int step = GROUP_ROUNDS / 2; step >= 1; step >>= 1)
                if (rank >= tot - plan->rem[d + step][c]) d += step;
            const uint32_t g = plan->gbase[d][c] + (rank - (tot - plan->rem[d][c]));
            slot = c & 3u;
            u = residue_group_place(g, lg, dm1, blocks_of_16);
        } else {
            const uint32_t li = plan->lbase[c] + (rank - (tot - left));
            const uint32_t jg = li % lg;
            slot = li / lg;
            u = leftover_group_place(jg, gtot, lg, dm1, blocks_of_16);
        }
        const int64_t pos = blocks_of_16 ? group_slot_position16(u, slot) : group_slot_position(u, slot);
        if (pos < n_alloc) gc8[pos] = make_uint4(v.x, v.y, (uint32_t)i, 0u);
    }
    // holes (blocks of 16: every position was marked empty before this kernel ran)
    if (blockIdx.x == 0 && threadIdx.x < 32 && !blocks_of_16) {
        const int tid = threadIdx.x;
        const int64_t T = (int64_t)gtot + lg;
        int64_t pos = -1;
        if (tid < 4) {
            const uint32_t li = ltot + (uint32_t)tid;
            if (li < 4u * lg) {
                const uint32_t jg = li % lg;
                pos = group_slot_position(leftover_group_place(jg, gtot, lg, dm1, 0), li / lg);
            }
        } else if (tid < 8) {
            if (T & 1) pos = group_slot_position(T, (uint32_t)tid - 4);
        } else {
            pos = ((T + 1) >> 1) * 8 + (tid - 8);
        }
        if (pos >= 0 && pos < n_alloc) gc8[pos] = make_uint4(0u, 0u, ORIGIN_NONE, 0u);
    }
}

template <int R, int THREADS, int DEPTH>
__global__ __launch_bounds__(THREADS) void assign_scan8p_kernel(const uint8_t* __restrict__ codes, int64_t N,
                                                                const uint4* __restrict__ gc8,
                                                                const float4* __restrict__ img, int ntiles,
                                                                int32_t* __restrict__ assign,
                                                                float* __restrict__ dist, RankOut ro = RankOut{})
{
    constexpr int LPS = 4, TK = 16, M = 8;
    constexpr int SLOTS = THREADS / LPS;
    constexpr int C = SLOTS * R;
    constexpr int NF = TILE_F4 / THREADS;
    constexpr uint32_t PLANE = 16384;       // bytes per subspace plane: 256 subcodes x 16 centers
    static_assert(TILE_F4 % THREADS == 0, "tile must divide evenly over the workgroup");
    static_assert(R * THREADS * 8 <= TILE_BYTES, "the per-lane records must fit the tile buffer");

    __shared__ float4 tile[TILE_F4];
    const char* tb = reinterpret_cast<const char*>(tile);

    const int tid = threadIdx.x;
    const int q = tid % LPS;
    const int c = tid / LPS;
    const int64_t base = (int64_t)blockIdx.x * C;
    const uint32_t low15 = 0x7fffu;

    // per code four registers, register j a 15-bit field (byte offset x_j*64 + 16q of subspace j's piece in its
    // row) and a 17-bit field from bit 15 up (the same for subspace j + 4, plus 64 KB), so that every remaining
    // plane offset (0 to 3 planes of 16 KB) fits the DS immediate and each unpack is one full-rate instruction
    uint32_t fld[R][4];
    float best[R];
    int tix[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t n = base + (int64_t)r * SLOTS + c;
        if (n >= N) n = N - 1;
        uint32_t lo, hi;
        if (gc8) {
            const uint4 g = gc8[n];
            lo = g.x;
            hi = g.y;
        } else {
            const uint2 g = *reinterpret_cast<const uint2*>(codes + n * 8);
            lo = g.x;
            hi = g.y;
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const uint32_t xa = (lo >> (8 * w)) & 255u, xb = (hi >> (8 * w)) & 255u;
            fld[r][w] = ((xa << 6) | ((uint32_t)q << 4)) | ((((xb << 6) | ((uint32_t)q << 4)) + 65536u) << 15);
        }
        best[r] = INFINITY;
        tix[r] = -1;
    }

    const uint32_t lane_off = (uint32_t)tid * 16u;
    v4f* ltile = reinterpret_cast<v4f*>(tile);
    auto gload = [&](int t, int i) -> v4f {
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float4*>(img + (size_t)t * TILE_F4), 0, TILE_BYTES, 0x00020000);
        return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, i * THREADS * 16, 0));
    };
    v4f pf[NF];
#pragma unroll
    for (int i = 0; i < NF; ++i) pf[i] = gload(0, i);

    auto issue = [&](int step) -> float4 {
        const int r = step / M, m = step % M;
        const uint32_t ad = (m < 4) ? unpack_low15(low15, fld[r][m]) : unpack_high17(fld[r][m - 4]);
        return lds_read16(tb, ad + (uint32_t)(m & 3) * PLANE);
    };

    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NF; ++i) ltile[i * THREADS + tid] = pf[i];
        __syncthreads();
        const int tn = t + 1 < ntiles ? t + 1 : t;
        float4 ring[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) ring[d] = issue(d);
        float4 sa;
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int i = 0; i < NF; ++i)
                if ((i * R * 5) / (NF * 8) == r) pf[i] = gload(tn, i);
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const int step = M * r + m;
                const float4 cur = ring[step % DEPTH];
                if (step + DEPTH < M * R) ring[step % DEPTH] = issue(step + DEPTH);
                if (m == 0) {
                    sa = cur;
                } else {
                    sa.x = sa.x + cur.x; sa.y = sa.y + cur.y; sa.z = sa.z + cur.z; sa.w = sa.w + cur.w;
                }
                if (m == M - 1) {
                    const float m4 = min3_f32(sa.x, sa.y, sa.z);
                    const float nb = min3_f32(m4, sa.w, best[r]);
                    tix[r] = (nb < best[r]) ? t : tix[r];
                    best[r] = nb;
                }
            }
        }
    }

    // Epilogue, transposed through LDS as in assign_scan4p_kernel: lane l finishes the codes l, l + THREADS, ...
    constexpr int CPL = (R + 3) / 4;                // codes per lane (the last ones may be past C)
    __syncthreads();
    {
        float2* rec = reinterpret_cast<float2*>(tile);
#pragma unroll
        for (int r = 0; r < R; ++r)
            rec[(r * SLOTS + c) * 4 + q] = make_float2(best[r], __builtin_bit_cast(float, tix[r]));
    }
    __syncthreads();
    __amdgpu_buffer_rsrc_t rs_img = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float4*>(img), 0, (uint32_t)ntiles * (uint32_t)TILE_BYTES, 0x00020000);
    constexpr int TNONE = 0x7fffffff;
#pragma unroll 1
    for (int i0 = 0; i0 < CPL; ++i0) {
        const int j = i0 * THREADS + tid;
        int64_t n = base + j;
        const bool live = n < N && j < C;
        if (!live) n = N - 1;
        const float4 ra = lds_read16(tb, (uint32_t)j * 32u), rb = lds_read16(tb, (uint32_t)j * 32u + 16u);
        const float b0 = ra.x, b1 = ra.z, b2 = rb.x, b3 = rb.z;
        const int t0 = __builtin_bit_cast(int, ra.y), t1 = __builtin_bit_cast(int, ra.w);
        const int t2 = __builtin_bit_cast(int, rb.y), t3 = __builtin_bit_cast(int, rb.w);
        const float sm = __builtin_fminf(__builtin_fminf(b0, b1), __builtin_fminf(b2, b3));
        const int c0 = (b0 == sm && t0 >= 0) ? t0 : TNONE, c1 = (b1 == sm && t1 >= 0) ? t1 : TNONE;
        const int c2 = (b2 == sm && t2 >= 0) ? t2 : TNONE, c3 = (b3 == sm && t3 >= 0) ? t3 : TNONE;
        int tm = c0 < c1 ? c0 : c1;
        tm = tm < c2 ? tm : c2;
        tm = tm < c3 ? tm : c3;
        uint32_t cand = (uint32_t)(c0 == tm) | ((uint32_t)(c1 == tm) << 1) | ((uint32_t)(c2 == tm) << 2) |
                        ((uint32_t)(c3 == tm) << 3);
        if (tm == TNONE || !live) cand = 0u;
        uint32_t lo, hi, og;
        if (gc8) {
            const uint4 g = gc8[n];
            lo = g.x;
            hi = g.y;
            og = live ? g.z : ORIGIN_NONE;
        } else {
            const uint2 g = *reinterpret_cast<const uint2*>(codes + n * 8);
            lo = g.x;
            hi = g.y;
            og = live ? 0u : ORIGIN_NONE;
        }
        int bi = IDX_NONE;
        while (__any(cand != 0u)) {                 // one trip unless lane positions tie exactly
            const int qe = cand ? (int)__builtin_ctz(cand) : 0;
            const uint32_t tb0 = cand ? (uint32_t)tm * (uint32_t)TILE_BYTES + (uint32_t)qe * 16u : 0xfff00000u;
            v4f sv = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, tb0 + ((lo & 255u) << 6), 0, 0));
#pragma unroll
            for (int m = 1; m < M; ++m) {
                const uint32_t x = ((m < 4 ? lo : hi) >> (8 * (m & 3))) & 255u;
                sv = sv + __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, tb0 + (x << 6), m * PLANE, 0));
            }
            if (cand) {
                const int kb = tm * TK + qe * 4;
                int k = IDX_NONE;
                if (sv.w == sm) k = kb + 3;
                if (sv.z == sm) k = kb + 2;
                if (sv.y == sm) k = kb + 1;
                if (sv.x == sm) k = kb;
                bi = k < bi ? k : bi;
                cand &= cand - 1u;
            }
        }
        if (og != ORIGIN_NONE) {
            const int64_t dst = gc8 ? (int64_t)og : base + j;
            const int kw = (bi == IDX_NONE) ? 0 : bi;
            assign[dst] = kw;
            if (dist) dist[dst] = sm;
            if (ro.count) ro.rank[dst] = atomicAdd(&ro.count[kw], 1u);
        }
    }
}

// gc8[pos] = (0, 0, ORIGIN_NONE, 0) for every position: the two-lane-slot layout marks its holes before the scatter
__global__ __launch_bounds__(256) void code8_group_clear_kernel(uint4* __restrict__ gc8, int64_t n_alloc)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_alloc; i += (int64_t)gridDim.x * 256)
        gc8[i] = make_uint4(0u, 0u, 0xffffffffu, 0u);
}

// ---------------------------------------------------------------------------------------------
// M = 8 scan over residue-grouped codes with slots of two lanes (8 centers per lane): what
// assign_scan4q_kernel is to assign_scan4p_kernel.  Same image (img[tile][m][x][16]) and arithmetic as
// assign_scan8p_kernel; a lane reads, per subspace, the 16-byte piece of its slot's half of the 64-byte row and
// then (address ^ 32) the piece of the other half; even slots start with the lower half, odd slots with the upper;
// a workgroup of 512 threads holds 256 R codes per tile fill instead of 128 R.
// ---------------------------------------------------------------------------------------------
template <int R, int THREADS, int DEPTH>
__global__ __launch_bounds__(THREADS) void assign_scan8q_kernel(int64_t N, const uint4* __restrict__ gc8,
                                                                const float4* __restrict__ img, int ntiles,
                                                                int32_t* __restrict__ assign,
                                                                float* __restrict__ dist, RankOut ro)
{
    constexpr int LPS = 2, TK = 16, M = 8;
    constexpr int SLOTS = THREADS / LPS;
    constexpr int C = SLOTS * R;
    constexpr int NF = TILE_F4 / THREADS;
    constexpr uint32_t PLANE = 16384;       // bytes per subspace plane: 256 subcodes x 16 centers
    static_assert(TILE_F4 % THREADS == 0, "tile must divide evenly over the workgroup");
    static_assert(R * THREADS * 8 <= TILE_BYTES, "the per-lane records must fit the tile buffer");
    static_assert(R % 2 == 0, "the epilogue gives every lane R / 2 codes");

    __shared__ float4 tile[TILE_F4];
    const char* tb = reinterpret_cast<const char*>(tile);

    const int tid = threadIdx.x;
    const int q = tid & 1;
    const int c = tid >> 1;
    const uint32_t hq = ((uint32_t)(c & 1) << 5) | ((uint32_t)q << 4);
    const int64_t base = (int64_t)blockIdx.x * C;
    const uint32_t low15 = 0x7fffu;

    uint32_t fld[R][4];
    float best[R];
    int tix[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t n = base + (int64_t)r * SLOTS + c;
        if (n >= N) n = N - 1;
        const uint4 g = gc8[n];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const uint32_t xa = (g.x >> (8 * w)) & 255u, xb = (g.y >> (8 * w)) & 255u;
            fld[r][w] = ((xa << 6) | hq) | ((((xb << 6) | hq) + 65536u) << 15);
        }
        best[r] = INFINITY;
        tix[r] = -1;
    }

    const uint32_t lane_off = (uint32_t)tid * 16u;
    v4f* ltile = reinterpret_cast<v4f*>(tile);
    auto gload = [&](int t, int i) -> v4f {
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float4*>(img + (size_t)t * TILE_F4), 0, TILE_BYTES, 0x00020000);
        return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, i * THREADS * 16, 0));
    };
    v4f pf[NF];
#pragma unroll
    for (int i = 0; i < NF; ++i) pf[i] = gload(0, i);

    struct Pair { float4 a, b; };
    auto issue = [&](int step) -> Pair {
        const int r = step / M, m = step % M;
        const uint32_t ad = (m < 4) ? unpack_low15(low15, fld[r][m]) : unpack_high17(fld[r][m - 4]);
        const uint32_t po = (uint32_t)(m & 3) * PLANE;
        Pair p;
        p.a = lds_read16(tb, ad + po);
        p.b = lds_read16(tb, (ad ^ 32u) + po);
        return p;
    };

    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NF; ++i) ltile[i * THREADS + tid] = pf[i];
        __syncthreads();
        const int tn = t + 1 < ntiles ? t + 1 : t;
        Pair ring[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) ring[d] = issue(d);
        float4 sa, sb;
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int i = 0; i < NF; ++i)
                if ((i * R * 5) / (NF * 8) == r) pf[i] = gload(tn, i);
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const int step = M * r + m;
                const Pair cur = ring[step % DEPTH];
                if (step + DEPTH < M * R) ring[step % DEPTH] = issue(step + DEPTH);
                if (m == 0) {
                    sa = cur.a;
                    sb = cur.b;
                } else {
                    sa.x = sa.x + cur.a.x; sa.y = sa.y + cur.a.y; sa.z = sa.z + cur.a.z; sa.w = sa.w + cur.a.w;
                    sb.x = sb.x + cur.b.x; sb.y = sb.y + cur.b.y; sb.z = sb.z + cur.b.z; sb.w = sb.w + cur.b.w;
                }
                if (m == M - 1) {
                    float m8 = min3_f32(sa.x, sa.y, sa.z);
                    m8 = min3_f32(m8, sa.w, sb.x);
                    m8 = min3_f32(m8, sb.y, sb.z);
                    const float nb = min3_f32(m8, sb.w, best[r]);
                    tix[r] = (nb < best[r]) ? t : tix[r];
                    best[r] = nb;
                }
            }
        }
    }

    // Epilogue, transposed through LDS: lane l finishes the codes l, l + THREADS, ...
    constexpr int CPL = R / 2;
    __syncthreads();
    {
        float2* rec = reinterpret_cast<float2*>(tile);
#pragma unroll
        for (int r = 0; r < R; ++r)
            rec[(r * SLOTS + c) * 2 + q] = make_float2(best[r], __builtin_bit_cast(float, tix[r]));
    }
    __syncthreads();
    __amdgpu_buffer_rsrc_t rs_img = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float4*>(img), 0, (uint32_t)ntiles * (uint32_t)TILE_BYTES, 0x00020000);
    constexpr int TNONE = 0x7fffffff;
#pragma unroll 1
    for (int i0 = 0; i0 < CPL; ++i0) {
        const int jj = i0 * THREADS + tid;
        int64_t n = base + jj;
        const bool live = n < N;
        if (!live) n = N - 1;
        const float4 ra = lds_read16(tb, (uint32_t)jj * 16u);
        const float b0 = ra.x, b1 = ra.z;
        const int t0 = __builtin_bit_cast(int, ra.y), t1 = __builtin_bit_cast(int, ra.w);
        const float sm = __builtin_fminf(b0, b1);
        const int c0 = (b0 == sm && t0 >= 0) ? t0 : TNONE, c1 = (b1 == sm && t1 >= 0) ? t1 : TNONE;
        const int tm = c0 < c1 ? c0 : c1;
        uint32_t cand = (uint32_t)(c0 == tm) | ((uint32_t)(c1 == tm) << 1);
        if (tm == TNONE || !live) cand = 0u;
        const uint4 g = gc8[n];
        const uint32_t og = live ? g.z : ORIGIN_NONE;
        const uint32_t hs = (uint32_t)((jj % SLOTS) & 1);
        int bi = IDX_NONE;
        while (__any(cand != 0u)) {
            const uint32_t qe = cand ? (uint32_t)__builtin_ctz(cand) : 0u;
            const uint32_t pA = 2u * hs + qe, pB = 2u * (1u - hs) + qe;
            const uint32_t tb0 = cand ? (uint32_t)tm * (uint32_t)TILE_BYTES : 0xfff00000u;
            v4f sA, sB;
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const uint32_t x = ((m < 4 ? g.x : g.y) >> (8 * (m & 3))) & 255u;
                const uint32_t o = tb0 + (x << 6);
                const v4f vA = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o + pA * 16u, m * PLANE, 0));
                const v4f vB = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs_img, o + pB * 16u, m * PLANE, 0));
                if (m == 0) { sA = vA; sB = vB; }
                else { sA = sA + vA; sB = sB + vB; }
            }
            if (cand) {
                const int kA = tm * TK + (int)pA * 4, kB = tm * TK + (int)pB * 4;
                int k = IDX_NONE;
                auto take = [&](const v4f& v, int k0) {
                    int kk = IDX_NONE;
                    if (v.w == sm) kk = k0 + 3;
                    if (v.z == sm) kk = k0 + 2;
                    if (v.y == sm) kk = k0 + 1;
                    if (v.x == sm) kk = k0;
                    k = kk < k ? kk : k;
                };
                take(sA, kA); take(sB, kB);
                bi = k < bi ? k : bi;
                cand &= cand - 1u;
            }
        }
        if (og != ORIGIN_NONE) {
            const int kw = (bi == IDX_NONE) ? 0 : bi;
            assign[og] = kw;
            if (dist) dist[og] = sm;
            if (ro.count) ro.rank[og] = atomicAdd(&ro.count[kw], 1u);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Subspace-skewed scan for M = 8, 16, 32 (64-bit SIFT-like codes, CNN-feature codes; Sec. 4).
//
// All M subspaces of TK = 128/M centers are resident (x-major image: row (x, m) of TK*4 bytes at
// byte x*512 + m*TK*4), LPS = TK/4 lanes form a slot and each lane reads one 16-byte piece of
// its code's row per step.  A 16-lane LDS access group holds SL = 16/LPS slots; slot j of the
// group runs j subspaces behind (it reads m = i - j in step i), so the SL rows of one access sit
// at SL different 16*LPS-byte positions of the 256-byte bank line: no conflicts.  Steps in which
// a slot has no subspace (i < j or i >= M + j) read a line of -0.0 after the tile; the sum is a
// chain over all M + SL - 1 steps, and since x + (-0.0) = x bit for bit its value is exactly
// the ascending-m fp32 sum of Eq. 3.  The skew costs (SL-1)/M extra steps.
// Per code and lane the pre-scaled offsets of all steps are kept as 16-bit fields (unpacked by
// one SDWA shift per read); minimum tracking, prefetch of the next tile and the epilogue are
// those of the M = 4 kernels (the epilogue rebuilds its offsets from the code bytes).
// ---------------------------------------------------------------------------------------------
template <int M, int R, int THREADS, int DEPTH = 1>
__global__ __launch_bounds__(THREADS) void assign_scan_skew_kernel(const uint8_t* __restrict__ codes, int64_t N,
                                                                   const float4* __restrict__ img, int ntiles,
                                                                   int32_t* __restrict__ assign,
                                                                   float* __restrict__ dist)
{
    constexpr int TK = 128 / M, LPS = TK / 4, SL = 16 / LPS, STEPS = M + SL - 1;
    constexpr int RQ = LPS;                   // row size in 16-byte units
    constexpr int NFW = (STEPS + 1) / 2;      // registers of packed offsets per code
    constexpr int SLOTS = THREADS / LPS;
    constexpr int C = SLOTS * R;
    constexpr int NF = TILE_F4 / THREADS;
    constexpr uint32_t PAD = TILE_BYTES;
    static_assert(TILE_F4 % THREADS == 0, "tile must divide evenly over the workgroup");

    __shared__ float4 tile[TILE_F4 + 16];
    const char* tb = reinterpret_cast<const char*>(tile);

    const int tid = threadIdx.x;
    const int q = tid % LPS;
    const int c = tid / LPS;
    const int j = c % SL;                     // this slot runs j subspaces behind
    const int64_t base = (int64_t)blockIdx.x * C;
    const uint32_t four = 4;

    if (tid < 16) tile[TILE_F4 + tid] = make_float4(-0.0f, -0.0f, -0.0f, -0.0f);

    uint32_t fld[R][NFW];
    float best[R];
    int tix[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t n = base + (int64_t)r * SLOTS + c;
        if (n >= N) n = N - 1;
        const uint8_t* x = codes + n * M;
#pragma unroll
        for (int w = 0; w < NFW; ++w) fld[r][w] = 0u;
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
            const int mm = i - j;
            const bool real = mm >= 0 && mm < M;
            const uint32_t xv = real ? (uint32_t)x[mm] : 0u;
            const uint32_t pos = (uint32_t)((mm + SL) % SL);                    // bank position of the row
            const uint32_t f = real ? (xv * 32u + (uint32_t)mm * RQ + (uint32_t)q)
                                    : ((PAD >> 4) + pos * RQ + (uint32_t)q);
            fld[r][i / 2] |= (i & 1) ? (f << 16) : f;
        }
        best[r] = INFINITY;
        tix[r] = -1;
    }

    const uint32_t lane_off = (uint32_t)tid * 16u;
    v4f* ltile = reinterpret_cast<v4f*>(tile);
    auto gload = [&](int t, int i) -> v4f {
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float4*>(img + (size_t)t * TILE_F4), 0, TILE_BYTES, 0x00020000);
        return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, i * THREADS * 16, 0));
    };
    v4f pf[NF];
#pragma unroll
    for (int i = 0; i < NF; ++i) pf[i] = gload(0, i);

    auto issue = [&](int r, int i) -> float4 {
        const uint32_t ad = (i & 1) ? sdwa_shl_word1(four, fld[r][i / 2]) : sdwa_shl_word0(four, fld[r][i / 2]);
        return lds_read16(tb, ad);
    };

    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NF; ++i) ltile[i * THREADS + tid] = pf[i];
        __syncthreads();
        // the loads of the next tile are spread over the first 5/8 of the scan (a burst of them would hold every
        // wave in the vector-memory queue while the LDS pipe idles); the reads of the next DEPTH steps are in
        // flight while the current one is added
        const int tn = t + 1 < ntiles ? t + 1 : t;
        float4 ring[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) ring[d] = issue(d / STEPS, d % STEPS);
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int i = 0; i < NF; ++i)
                if ((i * R * 5) / (NF * 8) == r) pf[i] = gload(tn, i);
            float4 sa;
#pragma unroll
            for (int i = 0; i < STEPS; ++i) {
                const int step = r * STEPS + i;
                const float4 cur = ring[step % DEPTH];
                if (step + DEPTH < R * STEPS) ring[step % DEPTH] = issue((step + DEPTH) / STEPS, (step + DEPTH) % STEPS);
                if (i == 0) {
                    sa = cur;
                } else {
                    sa.x = sa.x + cur.x; sa.y = sa.y + cur.y; sa.z = sa.z + cur.z; sa.w = sa.w + cur.w;
                }
            }
            const float m4 = min3_f32(sa.x, sa.y, sa.z);
            const float nb = min3_f32(m4, sa.w, best[r]);
            tix[r] = (nb < best[r]) ? t : tix[r];
            best[r] = nb;
        }
    }

    // Epilogue: the lanes holding their slot's minimum re-read their 4 sums in the winning tile from
    // the image (offsets rebuilt from the code bytes), pick the first center attaining the minimum,
    // and the slot's lanes are merged by (value, index).
#pragma unroll 1
    for (int r0 = 0; r0 < R; ++r0) {
        float b = INFINITY;
        int tx = -1;
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (r == r0) { b = best[r]; tx = tix[r]; }
        float smin = b;
#pragma unroll
        for (int d = LPS / 2; d >= 1; d >>= 1) smin = __builtin_fminf(smin, __shfl_xor(smin, d));
        const bool need = tx >= 0 && b == smin;
        int bi = IDX_NONE;
        float bv = INFINITY;
        int64_t n = base + (int64_t)r0 * SLOTS + c;
        if (need) {
            const int64_t nn = n < N ? n : N - 1;
            const uint8_t* x = codes + nn * M;
            const char* gbase = reinterpret_cast<const char*>(img + (size_t)tx * TILE_F4);
            v4f sv = *reinterpret_cast<const v4f*>(gbase + (uint32_t)x[0] * 512u + (uint32_t)q * 16u);
#pragma unroll 4
            for (int m = 1; m < M; ++m)
                sv = sv + *reinterpret_cast<const v4f*>(gbase + (uint32_t)x[m] * 512u + (uint32_t)(m * RQ + q) * 16u);
            const int kb = tx * TK + q * 4;
            bv = b;
            if (sv.w == b) { bi = kb + 3; bv = sv.w; }
            if (sv.z == b) { bi = kb + 2; bv = sv.z; }
            if (sv.y == b) { bi = kb + 1; bv = sv.y; }
            if (sv.x == b) { bi = kb; bv = sv.x; }
        }
#pragma unroll
        for (int d = LPS / 2; d >= 1; d >>= 1) {
            float ob = __shfl_xor(bv, d);
            int oi = __shfl_xor(bi, d);
            if (ob < bv || (ob == bv && oi < bi)) { bv = ob; bi = oi; }
        }
        if (q == 0 && n < N) {
            assign[n] = (bi == IDX_NONE) ? 0 : bi;
            if (dist) dist[n] = bv;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Sliding-window skewed scan for wide codes, M = 16, 32 (CNN-feature codes; Sec. 4).
//
// A tile is TK = 16 centers, and its M subspace planes (img[tile][s][x][16 centers], 16 KB each) do not
// fit the LDS together, so they pass through it: the LDS holds a ring of eight planes, interleaved per
// subcode -- row (x, s) of 64 bytes at byte x*512 + (s mod 8)*64, so that a row's bank quarter is s mod 4
// whatever x is -- and every phase four new planes replace the four oldest ones (64 KB per fill).  Per
// code and lane the eight partial sums of Eq. 3 stay in registers across the phases and are added to in
// ascending s, which keeps the bits of the sequential fp32 sum.
//
// Two lanes form a slot (one code) and own the row's four 16-byte pieces two each; a 16-lane LDS access
// holds eight slots.  Slot class j = 0..3 runs j subspaces behind (it reads s = 4*phase + t - j in step t
// of a phase), which puts the rows of the four classes in four different bank quarters, and of the two
// slots of a class one reads its lanes' lower pieces first and the other the upper: sixteen different
// 16-byte positions in every access, whatever the subcodes.  Because the ring holds three planes more
// than a phase consumes, a slot that runs behind still finds its planes: the skew costs three steps per
// code and TILE (35 steps for 32 subspaces: j steps of -0.0 reads before the first plane, 3 - j after the
// last), not per fill.
//
// What a lane reads in a phase -- four subcodes of its code, shifted by its slot's j -- comes from an
// array the host prepares once per launch (code_skew_kernel): S[phase][position] = those four bytes as one
// word, four bytes per code and phase.  The address of a read is (byte << 9) + a per-lane constant of the
// ring position.  Minimum tracking, tile prefetch and winner recovery are those of the other scans.
// ---------------------------------------------------------------------------------------------
template <int M>
__global__ __launch_bounds__(256) void code_skew_kernel(const uint8_t* __restrict__ codes, int64_t N,
                                                        uint32_t* __restrict__ S, int64_t n_alloc)
{
    constexpr int NW = M / 4, NPH = M / 4 + 1;
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= n_alloc) return;
    const int j = (int)((n & 7) >> 1);                  // the slot class of this position
    const int64_t src = n < N ? n : N - 1;              // positions past the end repeat the last code
    const uint32_t* cw = reinterpret_cast<const uint32_t*>(codes + src * M);
    uint32_t w[NW + 2];
    w[0] = 0u;
#pragma unroll
    for (int i = 0; i < NW; ++i) w[i + 1] = cw[i];
    w[NW + 1] = 0u;
#pragma unroll
    for (int ph = 0; ph < NPH; ++ph) {
        // bytes 4 ph - j .. 4 ph - j + 3 of the code (zero outside it)
        const unsigned long long pair = ((unsigned long long)w[ph + 1] << 32) | w[ph];
        S[(size_t)ph * n_alloc + n] = (uint32_t)(pair >> (8 * (4 - j)));
    }
}

template <int T_BYTE>
__device__ __forceinline__ uint32_t sdwa_shl_byte(uint32_t sh, uint32_t v)
{
    uint32_t r;
    if (T_BYTE == 0)
        asm volatile("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0"
                     : "=v"(r) : "v"(sh), "v"(v));
    else if (T_BYTE == 1)
        asm volatile("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1"
                     : "=v"(r) : "v"(sh), "v"(v));
    else if (T_BYTE == 2)
        asm volatile("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2"
                     : "=v"(r) : "v"(sh), "v"(v));
    else
        asm volatile("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3"
                     : "=v"(r) : "v"(sh), "v"(v));
    return r;
}

template <int M, int R, int THREADS, int DEPTH>
__global__ __launch_bounds__(THREADS) void assign_scan_sw_kernel(const uint8_t* __restrict__ codes, int64_t N,
                                                                 const uint32_t* __restrict__ S, int64_t n_alloc,
                                                                 const float4* __restrict__ img, int ntiles,
                                                                 int32_t* __restrict__ assign,
                                                                 float* __restrict__ dist, RankOut ro = RankOut{},
                                                                 int64_t first_workgroup = 0)
{
    constexpr int TK = 16, LPS = 2, NPH = M / 4 + 1;
    constexpr int SLOTS = THREADS / LPS;
    constexpr int C = SLOTS * R;
    constexpr int PLANE_F4 = 1024;                    // float4 per plane (256 subcodes x 16 centers)
    constexpr int NF = 4 * PLANE_F4 / THREADS;        // float4 per thread per fill (four planes)
    constexpr int SD = R;                             // the words of a whole phase are loaded one phase ahead
    constexpr uint32_t PAD = TILE_BYTES;              // 256 bytes of -0.0 after the ring
    constexpr int XR = THREADS / 16;                  // subcode rows one float4 per thread covers in a fill
    static_assert(THREADS == 512 || THREADS == 1024, "the fill mapping takes whole rows of 16 threads");
    static_assert(C % 8 == 0 && R % SD == 0, "slot classes repeat every 8 positions; the word ring holds SD codes");

    __shared__ float4 tile[TILE_F4 + 16];
    const char* tb = reinterpret_cast<const char*>(tile);

    const int tid = threadIdx.x;
    const int q = tid & 1;
    const int c = tid >> 1;
    const int j = (c & 7) >> 1;                       // subspaces this slot runs behind
    const int h = c & 1;                              // 1: the lanes read the upper of their two pieces first
    const int64_t base = ((int64_t)blockIdx.x + first_workgroup) * C;   // a launch may cover a stretch of the workgroups
    const uint32_t nine = 9;

    if (tid < 16) tile[TILE_F4 + tid] = make_float4(-0.0f, -0.0f, -0.0f, -0.0f);

    // ring position constants: a read of ring slot e (subspace s = e mod 8 for a slot with j = 0) goes, for this
    // lane, to ring slot (e - j) mod 8, piece 2q + h first
    uint32_t uc[4], un[4];                            // current phase (e = t or 4 + t), next phase
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        uc[t] = (uint32_t)((t - j) & 7) * 64u + (uint32_t)(2 * q + h) * 16u;
        un[t] = (uint32_t)((4 + t - j) & 7) * 64u + (uint32_t)(2 * q + h) * 16u;
    }

    float acc[R][8];
    float best[R];
    int tix[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[r][i] = -0.0f;
        best[r] = INFINITY;
        tix[r] = -1;
    }

    // fill: element e = i*THREADS + tid of the four planes is (x = e >> 4, plane e >> 2 & 3, piece e & 3): the 16
    // lanes of an LDS write cover four planes x four pieces of one x, sixteen different positions
    const uint32_t lds_w = (uint32_t)(tid >> 4) * 512u + (uint32_t)((tid >> 2) & 3) * 64u + (uint32_t)(tid & 3) * 16u;
    const uint32_t glb_r = (uint32_t)((tid >> 2) & 3) * 16384u + (uint32_t)(tid >> 4) * 64u + (uint32_t)(tid & 3) * 16u;
    auto gload = [&](int64_t plane0, int i) -> v4f {
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float4*>(img + (size_t)plane0 * PLANE_F4), 0, 4 * PLANE_F4 * 16, 0x00020000);
        return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, glb_r, i * XR * 64, 0));
    };
    v4f pf[NF];
#pragma unroll
    for (int i = 0; i < NF; ++i) pf[i] = gload(0, i);
    auto fill = [&](int half) {
        char* dst = reinterpret_cast<char*>(tile) + lds_w + (uint32_t)half * 256u;
#pragma unroll
        for (int i = 0; i < NF; ++i) *reinterpret_cast<v4f*>(dst + i * XR * 512) = pf[i];
    };

    // subcode words: S[phase][base + r*SLOTS + c], read through a buffer descriptor of the workgroup's stretch of
    // a phase (uniform base, one 32-bit lane offset, the code as a scalar offset: no 64-bit address per code)
    const uint32_t word_off = (uint32_t)c * 4u;
    auto wload = [&](const uint32_t* phase_words, int r) -> uint32_t {
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(phase_words), 0, C * 4,
                                                                      0x00020000);
        return __builtin_amdgcn_raw_buffer_load_b32(rs, word_off, r * SLOTS * 4, 0);
    };
    const uint32_t* sp = S + base;
    uint32_t sw[SD];
#pragma unroll
    for (int r = 0; r < SD; ++r) sw[r] = wload(sp, r);

    struct Pair { float4 a, b; };

    // One phase: KIND 0 = first of a tile (the slot's first j steps read -0.0), 1 = middle, 2 = last (3 steps; the
    // steps past the slot's last subspace read -0.0; ends with the minimum update).  `next_words` = the words of
    // the phase after this one; `pf_plane` >= 0: the four planes to prefetch for the next fill.
    auto scan_phase = [&](auto kind_c, const uint32_t* next_words, int64_t pf_plane, int t_index) {
        constexpr int KIND = decltype(kind_c)::value;
        constexpr int NS = KIND == 2 ? 3 : 4;
        auto issue = [&](int st) -> Pair {
            const int r = st / NS, t = st % NS;
            const uint32_t w = sw[r % SD];
            uint32_t ad = (t == 0) ? sdwa_shl_byte<0>(nine, w) : (t == 1) ? sdwa_shl_byte<1>(nine, w)
                        : (t == 2) ? sdwa_shl_byte<2>(nine, w) : sdwa_shl_byte<3>(nine, w);
            ad += uc[t];
            if (KIND == 0 && t < 3) ad = (j > t) ? PAD + (uc[t] & 255u) : ad;
            if (KIND == 2) ad = (j > t) ? ad : PAD + (uc[t] & 255u);
            Pair p;
            p.a = lds_read16(tb, ad);
            p.b = lds_read16(tb, ad ^ 16u);
            return p;
        };
        Pair ring[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) ring[d] = issue(d);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (KIND != 2) {
#pragma unroll
                for (int i = 0; i < NF; ++i)
                    if ((i * R * 5) / (NF * 8) == r) pf[i] = gload(pf_plane, i);
            }
#pragma unroll
            for (int t = 0; t < NS; ++t) {
                const int st = r * NS + t;
                const Pair cur = ring[st % DEPTH];
                if (st + DEPTH < R * NS) ring[st % DEPTH] = issue(st + DEPTH);
                acc[r][0] += cur.a.x; acc[r][1] += cur.a.y; acc[r][2] += cur.a.z; acc[r][3] += cur.a.w;
                acc[r][4] += cur.b.x; acc[r][5] += cur.b.y; acc[r][6] += cur.b.z; acc[r][7] += cur.b.w;
                if (t == NS - 1) {
                    // the word of code r is no longer needed (its last read was issued DEPTH steps ago)
                    sw[r % SD] = (r + SD < R) ? wload(sp, r + SD) : wload(next_words, r + SD - R);
                    if (KIND == 2) {
                        float m8 = min3_f32(acc[r][0], acc[r][1], acc[r][2]);
                        m8 = min3_f32(m8, acc[r][3], acc[r][4]);
                        m8 = min3_f32(m8, acc[r][5], acc[r][6]);
                        const float nb = min3_f32(m8, acc[r][7], best[r]);
                        tix[r] = (nb < best[r]) ? t_index : tix[r];
                        best[r] = nb;
#pragma unroll
                        for (int i = 0; i < 8; ++i) acc[r][i] = -0.0f;
                    }
                }
            }
        }
    };

    for (int t = 0; t < ntiles; ++t) {
        const int64_t plane_t = (int64_t)t * M;
        const int tn = t + 1 < ntiles ? t + 1 : t;
        // phase 0: planes 0..3 into the lower half of the ring
        __syncthreads();
        fill(0);
        __syncthreads();
        sp = S + base;
        scan_phase(std::integral_constant<int, 0>{}, sp + (size_t)n_alloc, plane_t + 4, t);
#pragma unroll
        for (int i = 0; i < 4; ++i) { const uint32_t x = uc[i]; uc[i] = un[i]; un[i] = x; }
#pragma unroll 1
        for (int ph = 1; ph < NPH - 1; ++ph) {
            __syncthreads();
            fill(ph & 1);
            __syncthreads();
            sp = S + (size_t)ph * n_alloc + base;
            const uint32_t* nxt = S + (size_t)(ph + 1) * n_alloc + base;
            const int64_t pfp = (ph + 1 < NPH - 1) ? plane_t + 4 * (ph + 1) : (int64_t)tn * M;
            scan_phase(std::integral_constant<int, 1>{}, nxt, pfp, t);
#pragma unroll
            for (int i = 0; i < 4; ++i) { const uint32_t x = uc[i]; uc[i] = un[i]; un[i] = x; }
        }
        // last phase: no new planes; the slots that run behind finish their last subspaces
        sp = S + (size_t)(NPH - 1) * n_alloc + base;
        scan_phase(std::integral_constant<int, 2>{}, S + base, (int64_t)-1, t);
    }

    // Epilogue: the lanes holding their slot's minimum rebuild the sums of their 8 centers in the winning tile
    // from the image in global memory (same bits, same order of additions), pick the lowest center attaining the
    // minimum, and the two lanes of the slot are merged by (value, index).
    const int p1 = 2 * q + h, p2 = p1 ^ 1;
#pragma unroll 1
    for (int r0 = 0; r0 < R; ++r0) {
        float b = INFINITY;
        int tx = -1;
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (r == r0) { b = best[r]; tx = tix[r]; }
        const float smin = __builtin_fminf(b, __shfl_xor(b, 1));
        const bool need = tx >= 0 && b == smin;
        int bi = IDX_NONE;
        float bv = INFINITY;
        const int64_t n = base + (int64_t)r0 * SLOTS + c;
        if (need) {
            const int64_t nn = n < N ? n : N - 1;
            const uint8_t* x = codes + nn * M;
            const char* gbase = reinterpret_cast<const char*>(img + (size_t)tx * M * PLANE_F4);
            v4f sa = *reinterpret_cast<const v4f*>(gbase + (uint32_t)x[0] * 64u + (uint32_t)p1 * 16u);
            v4f sb = *reinterpret_cast<const v4f*>(gbase + (uint32_t)x[0] * 64u + (uint32_t)p2 * 16u);
#pragma unroll 4
            for (int s = 1; s < M; ++s) {
                const char* row = gbase + (size_t)s * 16384 + (uint32_t)x[s] * 64u;
                sa = sa + *reinterpret_cast<const v4f*>(row + (uint32_t)p1 * 16u);
                sb = sb + *reinterpret_cast<const v4f*>(row + (uint32_t)p2 * 16u);
            }
            const int ka = tx * TK + p1 * 4, kb = tx * TK + p2 * 4;
            int k = IDX_NONE;
            if (sa.w == b) k = ka + 3;
            if (sa.z == b) k = ka + 2;
            if (sa.y == b) k = ka + 1;
            if (sa.x == b) k = ka;
            int k2 = IDX_NONE;
            if (sb.w == b) k2 = kb + 3;
            if (sb.z == b) k2 = kb + 2;
            if (sb.y == b) k2 = kb + 1;
            if (sb.x == b) k2 = kb;
            bi = k < k2 ? k : k2;
            bv = b;
        }
        {
            const float ob = __shfl_xor(bv, 1);
            const int oi = __shfl_xor(bi, 1);
            if (ob < bv || (ob == bv && oi < bi)) { bv = ob; bi = oi; }
        }
        if (q == 0 && n < N) {
            const int kw = (bi == IDX_NONE) ? 0 : bi;
            assign[n] = kw;
            if (dist) dist[n] = bv;
            if (ro.count) ro.rank[n] = atomicAdd(&ro.count[kw], 1u);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Zero fill (a kernel, not a memset node, so that callers may capture the calls in a graph).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void zero_u32_kernel(uint32_t* __restrict__ p, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * 256;
    for (; i < n; i += stride) p[i] = 0u;
}

// ---------------------------------------------------------------------------------------------
// Eq. 7, atomic path: hist[k][m][j] += 1 for every code n with assign[n] = k, codes[n][m] = j.
// Integer atomics: exact and independent of order.  One lane per code.  Used when the number of
// centers is too large for the owner path below; hist must be zero on entry.  Cluster sizes are
// not counted here: the vote derives them from the histogram (sum over the bins of a subspace).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void histogram_atomic_kernel(const uint8_t* __restrict__ codes, int64_t N, int M,
                                                               const int32_t* __restrict__ assign, int K,
                                                               uint32_t* __restrict__ hist)
{
    int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    int k = assign[n];
    if ((unsigned)k >= (unsigned)K) return;
    const uint8_t* x = codes + n * M;
    uint32_t* h = hist + (size_t)k * M * L;
    if ((M & 3) == 0 && ((uintptr_t)codes & 3) == 0) {
        const uint32_t* xw = reinterpret_cast<const uint32_t*>(x);
        for (int w = 0; w < M / 4; ++w) {
            uint32_t p = xw[w];
            atomicAdd(&h[(size_t)(4 * w + 0) * L + (p & 255u)], 1u);
            atomicAdd(&h[(size_t)(4 * w + 1) * L + ((p >> 8) & 255u)], 1u);
            atomicAdd(&h[(size_t)(4 * w + 2) * L + ((p >> 16) & 255u)], 1u);
            atomicAdd(&h[(size_t)(4 * w + 3) * L + (p >> 24)], 1u);
        }
    } else {
        for (int m = 0; m < M; ++m) atomicAdd(&h[(size_t)m * L + x[m]], 1u);
    }
}

// ---------------------------------------------------------------------------------------------
// Eq. 7, sorted path (many centers): the code indices are first sorted by cluster with a counting
// sort (cluster sizes, exclusive prefix, scatter: one global atomic per code instead of one per
// code and subspace), then a workgroup owns KT consecutive clusters, reads their codes from the
// contiguous stretch of the sorted index array and counts into LDS; the private histograms are
// the result (written whole: no clearing pass, no global atomics on bins).  Out-of-range
// assignments are dropped by the sort.  The order of the indices inside a cluster depends on the
// atomics; counts do not.
// ---------------------------------------------------------------------------------------------
constexpr int SEG_COUNT_LDS_K = 16384;      // cluster sizes are counted in LDS up to this many clusters

__global__ __launch_bounds__(1024) void seg_count_kernel(const int32_t* __restrict__ assign, int64_t N, int K,
                                                         uint32_t* __restrict__ cnt)
{
    __shared__ uint32_t h[SEG_COUNT_LDS_K];
    const bool lds = K <= SEG_COUNT_LDS_K;
    if (lds) {
        for (int k = threadIdx.x; k < K; k += 1024) h[k] = 0u;
        __syncthreads();
    }
    for (int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x; i < N; i += (int64_t)gridDim.x * 1024) {
        const int k = assign[i];
        if ((unsigned)k < (unsigned)K) atomicAdd(lds ? &h[k] : &cnt[k], 1u);
    }
    if (lds) {
        __syncthreads();
        for (int k = threadIdx.x; k < K; k += 1024)
            if (h[k]) atomicAdd(&cnt[k], h[k]);
    }
}

// one workgroup: start[0..K] = exclusive prefix of cnt, cursor[0..K) = 0
__global__ __launch_bounds__(1024) void seg_prefix_kernel(const uint32_t* __restrict__ cnt, int K,
                                                          uint32_t* __restrict__ start, uint32_t* __restrict__ cursor)
{
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = 0u;
    __syncthreads();
    for (int k0 = 0; k0 < K; k0 += 1024) {
        const int k = k0 + tid;
        const uint32_t v = k < K ? cnt[k] : 0u;
        const uint32_t inc = wave_inclusive_scan(v);
        if ((tid & 63) == 63) wsum[tid >> 6] = inc;
        __syncthreads();
        uint32_t e = carry + inc - v;
        for (int w = 0; w < (tid >> 6); ++w) e += wsum[w];
        if (k < K) {
            start[k] = e;
            cursor[k] = 0u;
        }
        __syncthreads();
        if (tid == 1023) carry = e + v;
        __syncthreads();
    }
    if (tid == 0) start[K] = carry;
}

__global__ __launch_bounds__(256) void seg_scatter_kernel(const int32_t* __restrict__ assign, int64_t N, int K,
                                                          const uint32_t* __restrict__ start,
                                                          uint32_t* __restrict__ cursor, uint32_t* __restrict__ sidx)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < N; i += (int64_t)gridDim.x * 256) {
        const int k = assign[i];
        if ((unsigned)k < (unsigned)K) sidx[start[k] + atomicAdd(&cursor[k], 1u)] = (uint32_t)i;
    }
}

// the scatter when the scan has left every code's rank inside its cluster: no atomics, one pass
__global__ __launch_bounds__(256) void seg_place_kernel(const int32_t* __restrict__ assign,
                                                        const uint32_t* __restrict__ rank, int64_t N, int K,
                                                        const uint32_t* __restrict__ start, uint32_t* __restrict__ sidx)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < N; i += (int64_t)gridDim.x * 256) {
        const int k = assign[i];
        if ((unsigned)k < (unsigned)K) sidx[start[k] + rank[i]] = (uint32_t)i;
    }
}

// workgroup b owns clusters b*KT .. b*KT+KT-1; LDS holds KT*M*256 counters (at most HIST_LDS_WORDS)
__global__ __launch_bounds__(1024) void seg_hist_kernel(const uint8_t* __restrict__ codes, int M,
                                                        const uint32_t* __restrict__ start,
                                                        const uint32_t* __restrict__ sidx, int K, int KT,
                                                        uint32_t* __restrict__ hist)
{
    __shared__ uint32_t lh[32768];
    __shared__ uint32_t st[130];
    const int tid = threadIdx.x;
    const int k0 = blockIdx.x * KT;
    const int nk = K - k0 < KT ? K - k0 : KT;
    const int words = nk * M * L;
    for (int i = tid; i < words; i += 1024) lh[i] = 0u;
    for (int i = tid; i <= nk; i += 1024) st[i] = start[k0 + i];
    __syncthreads();
    const uint32_t p0 = st[0], p1 = st[nk];
    const bool wordwise = (M & 3) == 0 && ((uintptr_t)codes & 3) == 0;
    for (uint32_t p = p0 + tid; p < p1; p += 1024) {
        // the cluster of position p: the last kk with st[kk] <= p
        int kk = 0;
        for (int step = 64; step >= 1; step >>= 1)
            if (kk + step < nk && st[kk + step] <= p) kk += step;
        const uint8_t* x = codes + (size_t)sidx[p] * M;
        uint32_t* h = lh + kk * M * L;
        if (wordwise) {
            const uint32_t* xw = reinterpret_cast<const uint32_t*>(x);
            for (int w = 0; w < M / 4; ++w) {
                const uint32_t v = xw[w];
                atomicAdd(&h[(4 * w + 0) * L + (v & 255u)], 1u);
                atomicAdd(&h[(4 * w + 1) * L + ((v >> 8) & 255u)], 1u);
                atomicAdd(&h[(4 * w + 2) * L + ((v >> 16) & 255u)], 1u);
                atomicAdd(&h[(4 * w + 3) * L + (v >> 24)], 1u);
            }
        } else {
            for (int m = 0; m < M; ++m) atomicAdd(&h[m * L + x[m]], 1u);
        }
    }
    __syncthreads();
    uint32_t* out = hist + (size_t)k0 * M * L;
    for (int i = tid; i < words; i += 1024) out[i] = lh[i];
}

// ---------------------------------------------------------------------------------------------
// Eq. 6, the naive update (kept as the comparison the paper measures sparse voting against): for
// every cluster and subspace all 256 candidates are tested against all members,
//   cost[k][m][l] = sum over members n of A^m[x_n^m][l],   centers[k][m] = argmin_l cost (lowest l),
// O(L M N) table entries.  Workgroup (k, m), thread = candidate l: the members' indices come from
// the same counting sort as the sorted-path histogram, each member contributes one 1 KB table
// row (a coalesced read), sums are fp64.  The order of the members inside a cluster is whatever
// the sort's atomics left, so the sums are reproducible only up to fp64 rounding (exactly, when
// the table entries are integers).  Empty clusters keep their code.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void naive_update_kernel(const uint8_t* __restrict__ codes, int M,
                                                           const uint32_t* __restrict__ start,
                                                           const uint32_t* __restrict__ sidx,
                                                           const float* __restrict__ tables,
                                                           uint8_t* __restrict__ centers, double* __restrict__ cost_out)
{
    __shared__ double sv[256];
    __shared__ int si[256];
    const int k = blockIdx.x, m = blockIdx.y, l = threadIdx.x;
    const uint32_t p0 = start[k], p1 = start[k + 1];
    const float* A = tables + (size_t)m * L * L;
    double acc = 0.0;
    for (uint32_t p = p0; p < p1; ++p) {
        const uint32_t x = codes[(size_t)sidx[p] * M + m];
        acc = acc + (double)A[x * L + l];
    }
    if (cost_out) cost_out[((size_t)k * M + m) * L + l] = acc;
    if (p0 == p1) return;                            // wave-uniform: the whole workgroup leaves
    sv[l] = acc;
    si[l] = l;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if (l < off) {
            const double ov = sv[l + off];
            const int oi = si[l + off];
            if (ov < sv[l] || (ov == sv[l] && oi < si[l])) {
                sv[l] = ov;
                si[l] = oi;
            }
        }
        __syncthreads();
    }
    if (l == 0) centers[(size_t)k * M + m] = (uint8_t)si[0];
}

// ---------------------------------------------------------------------------------------------
// Eq. 7, owner path: LDS-privatised histograms, no global atomics.
//
// Clusters are grouped KT at a time, KT chosen so that there are up to 255 groups (about one
// per CU) and KT*M*1 KB of histograms fit the LDS budget (16 KB or 128 KB).  A first kernel
// writes one byte per code, the group of its cluster (255 = none).  Workgroup (g, s) then owns
// group g and the s-th of S slices of the codes: it streams its slice of the group bytes with
// 16-byte loads (16 codes per lane and load; the byte array is small enough to stay in the
// XCD's L2 while all groups stream it), pushes the indices of the matching codes to an LDS
// queue, and after every batch the whole workgroup drains the queue -- one code per lane: load
// its assignment and subcodes, increment the private histograms with LDS atomics.  The private
// copy is stored whole (zeros included, so nothing needs clearing): with S = 1 it IS the result;
// with S > 1 slice s goes to its own partial array out + s*part_stride and the vote kernel adds
// the partials when it loads a histogram.
// ---------------------------------------------------------------------------------------------
constexpr int HIST_LDS_WORDS = 32768;   // 128 KB of private histograms (large instantiation)
constexpr int HIST_LDS_WORDS_SMALL = 4096;   // 16 KB (small instantiation: several workgroups per CU)
constexpr int HIST_QCAP = 4096;         // queue entries (16 KB)

// One code into the private histograms of its cluster (LDS atomics).  Kept out of line: it is called
// from many places of the scan loop, most of them cold.
__device__ __noinline__ void hist_add_code(uint32_t* lh, const uint8_t* __restrict__ codes,
                                           const int32_t* __restrict__ assign, int64_t n, int M, int k0, int kt,
                                           bool wide)
{
    int kk = assign[n] - k0;
    if ((unsigned)kk >= (unsigned)kt) return;
    uint32_t* h = lh + (size_t)kk * M * L;
    const uint8_t* x = codes + n * M;
    if (wide) {
        const uint32_t* xw = reinterpret_cast<const uint32_t*>(x);
        for (int w = 0; w < M / 4; ++w) {
            uint32_t p = xw[w];
            atomicAdd(&h[(4 * w + 0) * L + (p & 255u)], 1u);
            atomicAdd(&h[(4 * w + 1) * L + ((p >> 8) & 255u)], 1u);
            atomicAdd(&h[(4 * w + 2) * L + ((p >> 16) & 255u)], 1u);
            atomicAdd(&h[(4 * w + 3) * L + (p >> 24)], 1u);
        }
    } else {
        for (int m = 0; m < M; ++m) atomicAdd(&h[m * L + x[m]], 1u);
    }
}

__global__ __launch_bounds__(256) void cluster_group_kernel(const int32_t* __restrict__ assign, int64_t N, int K,
                                                            int KT, uint8_t* __restrict__ gid)
{
    int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    int k = assign[n];
    gid[n] = ((unsigned)k < (unsigned)K) ? (uint8_t)(k / KT) : (uint8_t)255;
}

template <int LDS_WORDS>
__global__ __launch_bounds__(1024) void histogram_owner_kernel(const uint8_t* __restrict__ codes, int64_t N, int M,
                                                               const int32_t* __restrict__ assign,
                                                               const uint8_t* __restrict__ gid, int K, int KT,
                                                               int S, uint32_t* __restrict__ hist,
                                                               size_t part_stride)
{
    __shared__ uint32_t lh[LDS_WORDS];
    __shared__ uint32_t queue[HIST_QCAP];
    __shared__ uint32_t qn;
    const int tid = threadIdx.x;
    const int g = blockIdx.x / S, s = blockIdx.x % S;
    const int k0 = g * KT;
    const int kt = (K - k0 < KT) ? K - k0 : KT;
    const int words = kt * M * L;
    for (int i = tid; i < words; i += 1024) lh[i] = 0u;
    if (tid == 0) qn = 0u;
    __syncthreads();

    // slice [lo, hi) of the codes, cut at multiples of 16 so that 16-byte loads of gid stay aligned
    const int64_t lo = (N * s / S) & ~(int64_t)15;
    const int64_t hi = (s + 1 == S) ? N : ((N * (s + 1) / S) & ~(int64_t)15);
    const bool wide = (M & 3) == 0 && ((uintptr_t)codes & 3) == 0;
    auto add_code = [&](int64_t n) { hist_add_code(lh, codes, assign, n, M, k0, kt, wide); };
    auto push = [&](int64_t n) {
        uint32_t slot = atomicAdd(&qn, 1u);
        if (slot < (uint32_t)HIST_QCAP) queue[slot] = (uint32_t)(n - lo);
        else add_code(n);                                  // queue full: count it right away
    };
    // drain(): the whole workgroup empties the queue, one code per lane.  Collective (barriers inside).
    auto drain = [&]() {
        const uint32_t cnt = qn < (uint32_t)HIST_QCAP ? qn : (uint32_t)HIST_QCAP;
        for (uint32_t i = tid; i < cnt; i += 1024) add_code(lo + queue[i]);
        __syncthreads();
        if (tid == 0) qn = 0u;
        __syncthreads();
    };

    const int64_t hi16 = lo + ((hi - lo) & ~(int64_t)15);
    const uint32_t gg = (uint32_t)g * 0x01010101u;
    if (((uintptr_t)gid & 15) == 0 && hi - lo < ((int64_t)1 << 32)) {
        constexpr int UNR = 8;
        const uint4* g4 = reinterpret_cast<const uint4*>(gid);
        const int64_t v_lo = lo / 16, v_hi = hi16 / 16;
        auto fetch = [&](int64_t vb, uint4 (&w)[UNR]) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                int64_t vi = vb + (int64_t)u * 1024 + tid;
                w[u] = (vi < v_hi) ? g4[vi] : make_uint4(~0u, ~0u, ~0u, ~0u);
            }
        };
        // Batches are visited in a rotated order that differs from group to group, so that the
        // workgroups, which all stream the same bytes, do not all ask the same L2 channel at once.
        const int64_t nbatch = (v_hi - v_lo + (int64_t)1024 * UNR - 1) / ((int64_t)1024 * UNR);
        const int64_t rot = nbatch > 0 ? ((int64_t)g * 7 + s) % nbatch : 0;
        auto batch_base = [&](int64_t b) { return v_lo + ((b + rot) % nbatch) * (int64_t)1024 * UNR; };
        uint4 w[UNR], wn[UNR];
        if (nbatch > 0) fetch(batch_base(0), wn);
        for (int64_t b = 0; b < nbatch; ++b) {                               // uniform trip count: barriers inside
            const int64_t vb = batch_base(b);
#pragma unroll
            for (int u = 0; u < UNR; ++u) w[u] = wn[u];
            if (b + 1 < nbatch) fetch(batch_base(b + 1), wn);                // next batch in flight
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int64_t n0 = (vb + (int64_t)u * 1024 + tid) * 16;
                // bit 8*b + j of mm is set iff byte b of word j equals g (exact zero-byte test per word)
                auto zb = [&](uint32_t word) -> uint32_t {
                    uint32_t x = word ^ gg;
                    return ~(((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x | 0x7f7f7f7fu);     // 0x80 in every zero byte
                };
                uint32_t mm = (zb(w[u].x) >> 7) | (zb(w[u].y) >> 6) | (zb(w[u].z) >> 5) | (zb(w[u].w) >> 4);
                while (mm) {                                                // 0 or 1 iterations for most lanes
                    const int bit = __ffs((int)mm) - 1;
                    mm &= mm - 1;
                    push(n0 + 4 * (bit & 7) + (bit >> 3));
                }
            }
            __syncthreads();
            if (qn >= (uint32_t)(HIST_QCAP / 2)) drain();                    // same value in every lane after the barrier
        }
    } else {
        for (int64_t nb = lo; nb < hi16; nb += 1024 * 4) {
            for (int u = 0; u < 4; ++u) {
                int64_t n = nb + (int64_t)u * 1024 + tid;
                if (n < hi16 && gid[n] == (uint8_t)g) push(n);
            }
            __syncthreads();
            if (qn >= (uint32_t)(HIST_QCAP / 2)) drain();
        }
    }
    __syncthreads();
    drain();
    for (int64_t n = hi16 + tid; n < hi; n += 1024)
        if (gid[n] == (uint8_t)g) add_code(n);
    __syncthreads();
    uint32_t* out = hist + (size_t)s * part_stride + (size_t)k0 * M * L;
    for (int i = tid; i < words; i += 1024) out[i] = lh[i];
}

// ---------------------------------------------------------------------------------------------
// Eq. 8: sparse vote with the table in LDS.
//
// A workgroup (1024 threads = 16 waves) serves one subspace m and CW consecutive clusters.  It
// holds half of A^m in LDS -- the rows A^m[j][.] of 128 member bins j, all 256 candidates l each
// (128 KB) -- and runs twice, once per half of the bins; the rows of the second half travel to
// registers while the first is in use.  A wave takes VOTE_CPW clusters per pass and keeps their
// 256 running sums in registers across the two halves: lane i owns the candidates 4i .. 4i+3,
// v accumulates in fp32 from 0 in ascending j with one fmaf per non-zero bin, exactly as Eq. 8 is
// read here, and every bin is visited once.  The non-zero bins are not compacted to a list: the
// wave walks the set bits of the ballot (h_j != 0) in ascending order, takes the count of bin j
// from its lane (a scalar), reads row j (one conflict-free 16-byte read per lane) and issues
// four fmaf.  The 256-way argmin is a per-lane ascending strict "<" and a (value, index)
// xor-shuffle merge, so the lowest index wins ties.  The cluster size is the sum of the bins
// (the same for every subspace): an empty cluster keeps its code, and subspace 0 stores the
// size to counts[k].  If the histogram arrives as S > 1 partial arrays they are added while
// loading (integer, exact) and the total is stored to hist.
// ---------------------------------------------------------------------------------------------
constexpr int VOTE_MAX_CW = 1024;        // clusters per workgroup
constexpr int VOTE_THREADS = 1024;       // 16 waves: many row reads in flight
constexpr int VOTE_WAVES = VOTE_THREADS / 64;
constexpr int VOTE_CPW = 2;              // clusters per wave whose sums are held in registers together

// REC: the histograms do not arrive from memory; the workgroup counts them itself, for its subspace, from the
// (code, center) records that the M = 4 scan filed by cluster group (its CW clusters are one group: CW = KT <=
// VOTE_REC_KT, the group's row of the segment table fits VOTE_REC_SEGS entries), and stores them to hist.
constexpr int VOTE_REC_KT = 16;
constexpr int VOTE_REC_SEGS = 1024;
struct VoteRecords {
    const uint2* pool;
    const uint2* seg;
    int nwg;
};

template <bool REC>
__global__ __launch_bounds__(VOTE_THREADS) void vote_kernel(uint32_t* __restrict__ hist,
                                                            const uint32_t* __restrict__ parts, int S,
                                                            size_t part_stride, uint32_t* __restrict__ counts,
                                                            int K, int M, int CW, const float* __restrict__ tables,
                                                            uint8_t* __restrict__ centers, VoteRecords vr)
{
    constexpr int NF = 8192 / VOTE_THREADS;     // float4 per thread per half of the table
    __shared__ float4 At[128 * 64];             // [row j of the half][lane: candidates 4 lane .. 4 lane + 3]
    __shared__ uint32_t lhist[REC ? VOTE_REC_KT * L : 1];     // REC: bins of the workgroup's clusters, this subspace
    __shared__ uint2 lseg[REC ? VOTE_REC_SEGS : 1];           // REC: the group's (first record, count) per scan workgroup
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int blocks_per_m = (K + CW - 1) / CW;
    const int m = blockIdx.x / blocks_per_m;
    const int c0 = (blockIdx.x % blocks_per_m) * CW;
    const int cn = (K - c0 < CW) ? K - c0 : CW;
    const v4f* A4v = reinterpret_cast<const v4f*>(tables + (size_t)m * L * L);        // row j = A4v[64 j .. 64 j + 63]
    v4f* Atv = reinterpret_cast<v4f*>(At);

    // bins chunk*64 + lane, chunk = 0..3, of one (cluster, subspace): the S <= 16 partial arrays are added, all
    // loads of a cluster in flight together (slices past S re-read the last one and are not added)
    auto load_bins = [&](size_t pair, uint32_t (&out)[4]) {
        if (REC) {
            const int cl = (int)(pair / (size_t)M) - c0;          // cluster inside the workgroup's group
#pragma unroll
            for (int chunk = 0; chunk < 4; ++chunk) out[chunk] = lhist[cl * L + chunk * 64 + lane];
            return;
        }
        const size_t at = pair * L + lane;
        if (S <= 1) {
#pragma unroll
            for (int chunk = 0; chunk < 4; ++chunk) out[chunk] = hist[at + chunk * 64];
            return;
        }
        uint32_t t[8][4];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t* src = parts + (size_t)(u < S ? u : S - 1) * part_stride + at;
#pragma unroll
            for (int chunk = 0; chunk < 4; ++chunk) t[u][chunk] = src[chunk * 64];
        }
#pragma unroll
        for (int chunk = 0; chunk < 4; ++chunk) {
            uint32_t sum = 0u;
#pragma unroll
            for (int u = 0; u < 8; ++u) sum += (u < S) ? t[u][chunk] : 0u;
            out[chunk] = sum;
        }
        if (S > 8) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t* src = parts + (size_t)(8 + u < S ? 8 + u : S - 1) * part_stride + at;
#pragma unroll
                for (int chunk = 0; chunk < 4; ++chunk) t[u][chunk] = src[chunk * 64];
            }
#pragma unroll
            for (int chunk = 0; chunk < 4; ++chunk) {
                uint32_t sum = 0u;
#pragma unroll
                for (int u = 0; u < 8; ++u) sum += (8 + u < S) ? t[u][chunk] : 0u;
                out[chunk] += sum;
            }
        }
    };
    // REC: Eq. 7 for this workgroup's clusters and subspace: the group's row of the segment table goes to LDS, then
    // a wave per stretch of records, sixteen stretches' loads in flight per wave, one LDS atomic per record.  This
    // runs before the table rows are requested: vector-memory results return in order, and the record loads would
    // otherwise wait behind 128 KB of table rows (measured: 3.5 us more per launch).
    auto count_from_records = [&]() {
        const int g = blockIdx.x % blocks_per_m;
        for (int i = tid; i < VOTE_REC_KT * L; i += VOTE_THREADS) lhist[i] = 0u;
        for (int i = tid; i < vr.nwg; i += VOTE_THREADS) lseg[i] = vr.seg[(size_t)g * vr.nwg + i];
        __syncthreads();
        const uint32_t sh = 8u * (uint32_t)m;
        constexpr int SB = 16;
        for (int w0 = wave; w0 < vr.nwg; w0 += SB * VOTE_WAVES) {
            uint2 sg[SB], r[SB];
#pragma unroll
            for (int u = 0; u < SB; ++u) {
                const int w = w0 + u * VOTE_WAVES;
                sg[u] = w < vr.nwg ? lseg[w] : make_uint2(0u, 0u);
                r[u] = (uint32_t)lane < sg[u].y ? vr.pool[(size_t)sg[u].x + lane] : make_uint2(0u, 0xffffffffu);
            }
#pragma unroll
            for (int u = 0; u < SB; ++u) {
                const uint32_t kk = r[u].y - (uint32_t)c0;
                if (kk < (uint32_t)cn) atomicAdd(&lhist[kk * L + ((r[u].x >> sh) & 255u)], 1u);
                // a stretch longer than a wave (a group holding most of a scan workgroup's codes)
                for (uint32_t i = lane + 64; i < sg[u].y; i += 64) {
                    const uint2 x = vr.pool[(size_t)sg[u].x + i];
                    const uint32_t k2 = x.y - (uint32_t)c0;
                    if (k2 < (uint32_t)cn) atomicAdd(&lhist[k2 * L + ((x.x >> sh) & 255u)], 1u);
                }
            }
        }
        __syncthreads();
    };

    auto fma_row = [](float4& acc, float h, const float4 r) {
        acc.x = fmaf(h, r.x, acc.x); acc.y = fmaf(h, r.y, acc.y);
        acc.z = fmaf(h, r.z, acc.z); acc.w = fmaf(h, r.w, acc.w);
    };

    if (REC) count_from_records();
    for (int b0 = 0; b0 < cn; b0 += VOTE_WAVES * VOTE_CPW) {
        v4f pf[NF];
#pragma unroll
        for (int i = 0; i < NF; ++i) pf[i] = A4v[i * VOTE_THREADS + tid];                  // rows 0 .. 127
        uint32_t hv[VOTE_CPW][4];
        float4 v[VOTE_CPW];
#pragma unroll
        for (int q = 0; q < VOTE_CPW; ++q) {
            const int c = b0 + q * VOTE_WAVES + wave;
            v[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (c < cn) {
                load_bins((size_t)(c0 + c) * M + m, hv[q]);
            } else {
#pragma unroll
                for (int chunk = 0; chunk < 4; ++chunk) hv[q][chunk] = 0u;
            }
        }
        // one half of the bins: fill the LDS rows from the registers, start the next half's loads, walk
        auto run_half = [&](auto half_c) {
            constexpr int half = decltype(half_c)::value;
            __syncthreads();                    // the rows in LDS are no longer being read
#pragma unroll
            for (int i = 0; i < NF; ++i) Atv[i * VOTE_THREADS + tid] = pf[i];
            __syncthreads();
            if (half == 0) {
#pragma unroll
                for (int i = 0; i < NF; ++i) pf[i] = A4v[8192 + i * VOTE_THREADS + tid];   // rows 128 .. 255
            }
#pragma unroll
            for (int q = 0; q < VOTE_CPW; ++q) {
#pragma unroll
                for (int ch = 0; ch < 2; ++ch) {
                    const uint32_t hb = hv[q][2 * half + ch];
                    const int hfi = __builtin_bit_cast(int, (float)hb);
                    uint64_t mask = __ballot(hb != 0u);
                    const float4* rows = At + ch * 64 * 64 + lane;
                    float4 acc = v[q];
                    int n = __popcll(mask);
                    for (; n >= 8; n -= 8) {                                 // eight rows in flight, fmas in order
                        int j[8];
                        float h[8];
                        float4 r[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            j[u] = __builtin_ctzll(mask);
                            mask &= mask - 1;
                            h[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(hfi, j[u]));
                            r[u] = rows[j[u] * 64];
                        }
                        __builtin_amdgcn_sched_barrier(0);                   // all eight reads before the first fmaf
#pragma unroll
                        for (int u = 0; u < 8; ++u) fma_row(acc, h[u], r[u]);
                    }
                    for (; n > 0; --n) {
                        const int j = __builtin_ctzll(mask);
                        mask &= mask - 1;
                        fma_row(acc, __builtin_bit_cast(float, __builtin_amdgcn_readlane(hfi, j)), rows[j * 64]);
                    }
                    v[q] = acc;
                }
            }
        };
        run_half(std::integral_constant<int, 0>{});
        run_half(std::integral_constant<int, 1>{});
#pragma unroll
        for (int q = 0; q < VOTE_CPW; ++q) {
            const int c = b0 + q * VOTE_WAVES + wave;
            if (c >= cn) continue;                                           // the same for the whole wave
            const size_t pair = (size_t)(c0 + c) * M + m;
            if (S > 1 || REC) {
#pragma unroll
                for (int chunk = 0; chunk < 4; ++chunk) hist[pair * L + chunk * 64 + lane] = hv[q][chunk];
            }
            uint32_t cnt = hv[q][0] + hv[q][1] + hv[q][2] + hv[q][3];
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) cnt += __shfl_xor(cnt, d);
            if (m == 0 && lane == 0) counts[c0 + c] = cnt;
            if (cnt == 0) continue;                                          // empty cluster keeps its code
            // Eq. 8's argmin as a sequential scan reads it: start from +inf, strict "<" over ascending l, so a
            // candidate whose sum is NaN or +inf is never taken and candidate 0 remains if none is
            float b = INFINITY;
            int bi = IDX_NONE;
            if (v[q].x < b) { b = v[q].x; bi = lane * 4; }
            if (v[q].y < b) { b = v[q].y; bi = lane * 4 + 1; }
            if (v[q].z < b) { b = v[q].z; bi = lane * 4 + 2; }
            if (v[q].w < b) { b = v[q].w; bi = lane * 4 + 3; }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                const float ob = __shfl_xor(b, d);
                const int oi = __shfl_xor(bi, d);
                if (ob < b || (ob == b && oi < bi)) { b = ob; bi = oi; }
            }
            if (lane == 0) centers[pair] = (uint8_t)(bi == IDX_NONE ? 0 : bi);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Exact index over the centers (Sec. 3.1, the table-based FindNN of Alg. 1).
//
// The paper's table is a hash table over the center codes that is probed with candidate codes in
// ascending distance until a stored one is met.  Here the centers are filed in 65536 buckets by their
// first two subcodes (c0, c1); a code (x0, x1, ...) walks the buckets in ascending A^0[x0][c0] and, inside,
// ascending A^1[x1][c1] -- two sorted rows -- and stops a walk as soon as a lower bound of everything
// that is left exceeds the best distance found.  The bound of a bucket is its partial sum continued with
// the smallest entry of the code's row in every remaining subspace, added in the order of Eq. 3: fp32
// addition is monotone in both operands, so the bound is never above the fp32 distance of any center of
// the bucket, the pruning is exact, and a NaN bound (comparisons false) prunes nothing.  Every visited
// center gets its full distance in the sequential order of Eq. 3; ties go to the lowest center index by
// comparing (distance, index), so the result is that of the linear scan bit for bit.
// One lane per code: the walks diverge, and every probe is a trip to memory rather than to the LDS.
// ---------------------------------------------------------------------------------------------
constexpr int INDEX_BUCKETS = 65536;

// grid (256, M), block 256: row x of A^m.  rowmin[m][x] = its smallest non-NaN entry (+inf if there is none);
// for m < 2 also ord[m][x][i] = the columns in ascending order of their entries (NaN last, ties by column)
__global__ __launch_bounds__(256) void index_rows_kernel(const float* __restrict__ tables, uint8_t* __restrict__ ord,
                                                         float* __restrict__ rowmin)
{
    __shared__ float row[L];
    __shared__ float red[4];
    const int x = blockIdx.x, m = blockIdx.y, c = threadIdx.x;
    const float v = tables[((size_t)m * L + x) * L + c];
    row[c] = v;
    float mn = (v != v) ? INFINITY : v;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) mn = __builtin_fminf(mn, __shfl_xor(mn, d));
    if ((c & 63) == 0) red[c >> 6] = mn;
    __syncthreads();
    if (c == 0) rowmin[m * L + x] = __builtin_fminf(__builtin_fminf(red[0], red[1]), __builtin_fminf(red[2], red[3]));
    if (m >= 2) return;
    const bool vnan = v != v;
    int rank = 0;
    for (int o = 0; o < L; ++o) {
        const float u = row[o];
        const bool unan = u != u;
        const bool before = (!unan && (vnan || u < v)) || ((u == v || (unan && vnan)) && o < c);
        rank += before ? 1 : 0;
    }
    ord[((size_t)m * L + x) * L + rank] = (uint8_t)c;
}

__global__ __launch_bounds__(256) void index_count_kernel(const uint8_t* __restrict__ centers, int K, int M,
                                                          uint32_t* __restrict__ cnt)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    atomicAdd(&cnt[(uint32_t)centers[(size_t)k * M] * 256u + centers[(size_t)k * M + 1]], 1u);
}

__global__ __launch_bounds__(256) void index_scatter_kernel(const uint8_t* __restrict__ centers, int K, int M,
                                                            const uint32_t* __restrict__ start,
                                                            uint32_t* __restrict__ cursor, uint32_t* __restrict__ items)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    const uint32_t b = (uint32_t)centers[(size_t)k * M] * 256u + centers[(size_t)k * M + 1];
    items[start[b] + atomicAdd(&cursor[b], 1u)] = (uint32_t)k;
}

__global__ __launch_bounds__(256) void assign_indexed_kernel(const uint8_t* __restrict__ codes, int64_t N, int M,
                                                             const uint8_t* __restrict__ centers,
                                                             const float* __restrict__ tables,
                                                             const uint8_t* __restrict__ ord,
                                                             const float* __restrict__ rowmin,
                                                             const uint32_t* __restrict__ start,
                                                             const uint32_t* __restrict__ items,
                                                             int32_t* __restrict__ assign, float* __restrict__ dist)
{
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    const uint8_t* x = codes + n * M;
    const int x0 = x[0], x1 = x[1];
    const float* A0 = tables + (size_t)x0 * L;
    const float* A1 = tables + ((size_t)L + x1) * L;
    const uint8_t* o0 = ord + (size_t)x0 * L;
    const uint8_t* o1 = ord + ((size_t)L + x1) * L;
    // what the subspaces 2 .. M-1 add at least, continued in the order of Eq. 3
    auto bound = [&](float p) -> float {
        for (int m = 2; m < M; ++m) p = p + rowmin[m * L + x[m]];
        return p;
    };
    float best = INFINITY;
    int bk = IDX_NONE;
    const float d1min = A1[o1[0]];
    for (int i = 0; i < L; ++i) {
        const int c0 = o0[i];
        const float d0 = A0[c0];
        if (bound(d0 + d1min) > best) break;                 // every later c0 has a larger bound
        for (int jj = 0; jj < L; ++jj) {
            const int c1 = o1[jj];
            const float p = d0 + A1[c1];
            if (bound(p) > best) break;                      // so has every later c1 under this c0
            const uint32_t b = (uint32_t)c0 * 256u + (uint32_t)c1;
            const uint32_t e1 = start[b + 1];
            for (uint32_t e = start[b]; e < e1; ++e) {
                const int k = (int)items[e];
                const uint8_t* mu = centers + (size_t)k * M;
                float sd = p;
                for (int m = 2; m < M; ++m) {
                    const float a = tables[((size_t)m * L + x[m]) * L + mu[m]];
                    sd = sd + a;
                }
                if (sd < best || (sd == best && bk != IDX_NONE && k < bk)) {
                    best = sd;
                    bk = k;
                }
            }
        }
    }
    assign[n] = (bk == IDX_NONE) ? 0 : bk;
    if (dist) dist[n] = best;
}

// ---------------------------------------------------------------------------------------------
// Per-iteration statistics of the convergence-checked loop (Alg. 1 with a stop condition).
// All reductions run in a fixed order (per-lane strided sums, xor-shuffle tree, per-block partials
// summed by one wave), so the fp64 objective is reproducible from run to run.
// ---------------------------------------------------------------------------------------------
constexpr int STAT_BLOCKS = 1024;

struct StatPartial { double dsum; unsigned long long cnt_a; unsigned long long cnt_b; };

__device__ __forceinline__ void stat_block_reduce(double d, unsigned long long a, unsigned long long b,
                                                  StatPartial* out)
{
    __shared__ StatPartial sm[4];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        d += __shfl_xor(d, o);
        a += __shfl_xor(a, o);
        b += __shfl_xor(b, o);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sm[wave].dsum = d; sm[wave].cnt_a = a; sm[wave].cnt_b = b; }
    __syncthreads();
    if (threadIdx.x == 0) {
        StatPartial r = sm[0];
        for (int w = 1; w < 4; ++w) { r.dsum += sm[w].dsum; r.cnt_a += sm[w].cnt_a; r.cnt_b += sm[w].cnt_b; }
        *out = r;
    }
}

// objective and number of changed assignments; also moves the new assignment into `prev`
__global__ __launch_bounds__(256) void iter_assign_stats_kernel(const int32_t* __restrict__ assign,
                                                                int32_t* __restrict__ prev,
                                                                const float* __restrict__ dist, int64_t N,
                                                                StatPartial* __restrict__ partial)
{
    double d = 0.0;
    unsigned long long changed = 0;
    for (int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x; n < N; n += (int64_t)STAT_BLOCKS * 256) {
        const int32_t a = assign[n];
        d += (double)dist[n];
        changed += (a != prev[n]);
        prev[n] = a;
    }
    stat_block_reduce(d, changed, 0ull, partial + blockIdx.x);
}

// non-zero histogram bins and non-empty clusters
__global__ __launch_bounds__(256) void iter_hist_stats_kernel(const uint32_t* __restrict__ hist, int64_t nbins,
                                                              const uint32_t* __restrict__ counts, int K,
                                                              StatPartial* __restrict__ partial)
{
    unsigned long long nz = 0, ne = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nbins; i += (int64_t)STAT_BLOCKS * 256)
        nz += (hist[i] != 0u);
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < K; k += (int64_t)STAT_BLOCKS * 256)
        ne += (counts[k] != 0u);
    stat_block_reduce(0.0, nz, ne, partial + blockIdx.x);
}

// out[0] = objective (as double bits), out[1] = changed, out[2] = nonzero bins, out[3] = nonempty
__global__ __launch_bounds__(64) void iter_stats_final_kernel(const StatPartial* __restrict__ pa,
                                                              const StatPartial* __restrict__ ph,
                                                              unsigned long long* __restrict__ out)
{
    double d = 0.0;
    unsigned long long ch = 0, nz = 0, ne = 0;
    for (int i = threadIdx.x; i < STAT_BLOCKS; i += 64) {
        d += pa[i].dsum;
        ch += pa[i].cnt_a;
        nz += ph[i].cnt_a;
        ne += ph[i].cnt_b;
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        d += __shfl_xor(d, o);
        ch += __shfl_xor(ch, o);
        nz += __shfl_xor(nz, o);
        ne += __shfl_xor(ne, o);
    }
    if (threadIdx.x == 0) {
        out[0] = (unsigned long long)__double_as_longlong(d);
        out[1] = ch;
        out[2] = nz;
        out[3] = ne;
    }
}

__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t* __restrict__ p, int64_t n, int32_t v)
{
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * 256;
    for (; i < n; i += stride) p[i] = v;
}

}  // namespace pqkm
