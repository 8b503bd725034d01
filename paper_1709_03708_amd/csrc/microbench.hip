// Microbenchmarks behind the roofline figures of the PQk-means scan on gfx950 (measurement code, not part of
// the method and not linked into libpqkm.so): LDS read and write rates, VALU issue rates of the instruction
// classes the scan uses, and the instruction mix of the M = 4 half-plane scan with and without a tile switch.
// One C entry point, pqkm_microbench(); `python bench.py --microbench` runs every test and prints the rates.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int LDS_BYTES = 128 * 1024;

__device__ inline uint32_t hash32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// ---------------------------------------------------------------------------------------------
// LDS reads: 8 independent reads in flight per lane, W bytes per lane.  LPR lanes share a row of
// LPR * W bytes; the rows sit at random positions of the 128 KB (LPR = 64: lane-consecutive).
// ---------------------------------------------------------------------------------------------
template <int W, int LPR>
__global__ __launch_bounds__(512) void lds_read_kernel(int iters, float* out, int salt)
{
    __shared__ float4 lds[LDS_BYTES / 16];
    for (int i = threadIdx.x; i < LDS_BYTES / 16; i += 512) lds[i] = make_float4(1.f, 2.f, 3.f, 4.f);
    __syncthreads();
    // the reads below are inline assembly with plain byte offsets: tell the compiler that the array is in use,
    // or it drops the allocation and the reads fall outside the (empty) LDS range
    asm volatile("" : : "v"(reinterpret_cast<uintptr_t>(&lds[threadIdx.x])) : "memory");
    const int tid = threadIdx.x;
    constexpr int ROWB = LPR * W;
    uint32_t a[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
        a[u] = (hash32((tid / LPR) * 2654435761u + u * 40503 + salt) % (LDS_BYTES / ROWB)) * ROWB + (tid % LPR) * W;
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        if (W == 16) {
            float4 r[8];
            asm volatile("ds_read_b128 %0, %8\n ds_read_b128 %1, %9\n ds_read_b128 %2, %10\n ds_read_b128 %3, %11\n"
                         "ds_read_b128 %4, %12\n ds_read_b128 %5, %13\n ds_read_b128 %6, %14\n ds_read_b128 %7, %15\n"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]),
                           "=&v"(r[7])
                         : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]));
            if (it == iters + 5) acc += r[0].x + r[7].w;       // never true: no arithmetic in the loop
        } else if (W == 8) {
            float2 r[8];
            asm volatile("ds_read_b64 %0, %8\n ds_read_b64 %1, %9\n ds_read_b64 %2, %10\n ds_read_b64 %3, %11\n"
                         "ds_read_b64 %4, %12\n ds_read_b64 %5, %13\n ds_read_b64 %6, %14\n ds_read_b64 %7, %15\n"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]),
                           "=&v"(r[7])
                         : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]));
            if (it == iters + 5) acc += r[0].x + r[7].y;
        } else {
            float r[8];
            asm volatile("ds_read_b32 %0, %8\n ds_read_b32 %1, %9\n ds_read_b32 %2, %10\n ds_read_b32 %3, %11\n"
                         "ds_read_b32 %4, %12\n ds_read_b32 %5, %13\n ds_read_b32 %6, %14\n ds_read_b32 %7, %15\n"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]),
                           "=&v"(r[7])
                         : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]));
            if (it == iters + 5) acc += r[0] + r[7];
        }
    }
    if (acc == 12345.678f) out[tid] = acc;
}

// LDS writes from registers: 128 KB per iteration, lane-consecutive 16-byte stores
__global__ __launch_bounds__(512) void lds_write_kernel(int iters, float* out)
{
    __shared__ float4 lds[LDS_BYTES / 16];
    const int tid = threadIdx.x;
    float4 v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = make_float4(tid + i, 1.f, 2.f, 3.f);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) lds[i * 512 + tid] = v[i];
#pragma unroll
        for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(v[i].x));
        __syncthreads();
    }
    if (lds[tid].x == 12345.678f) out[tid] = lds[tid + 1].y;
}

// ---------------------------------------------------------------------------------------------
// VALU issue rate: 16 independent chains per lane, 64 instructions per iteration, 1024 threads
// ---------------------------------------------------------------------------------------------
#define MB_OP16(INS, TAIL)                                                                                        \
    asm volatile(INS " %0, %16, %0 " TAIL "\n" INS " %1, %16, %1 " TAIL "\n" INS " %2, %16, %2 " TAIL "\n"       \
                 INS " %3, %16, %3 " TAIL "\n" INS " %4, %16, %4 " TAIL "\n" INS " %5, %16, %5 " TAIL "\n"       \
                 INS " %6, %16, %6 " TAIL "\n" INS " %7, %16, %7 " TAIL "\n" INS " %8, %16, %8 " TAIL "\n"       \
                 INS " %9, %16, %9 " TAIL "\n" INS " %10, %16, %10 " TAIL "\n" INS " %11, %16, %11 " TAIL "\n"   \
                 INS " %12, %16, %12 " TAIL "\n" INS " %13, %16, %13 " TAIL "\n" INS " %14, %16, %14 " TAIL "\n" \
                 INS " %15, %16, %15 " TAIL "\n"                                                                  \
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]), \
                   "+v"(a[8]), "+v"(a[9]), "+v"(a[10]), "+v"(a[11]), "+v"(a[12]), "+v"(a[13]), "+v"(a[14]),       \
                   "+v"(a[15])                                                                                    \
                 : "v"(b), "v"(c))
#define MB_SDWA "dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1"

template <int OP>
__global__ __launch_bounds__(1024) void valu_kernel(int iters, float* out)
{
    float a[16];
    for (int i = 0; i < 16; ++i) a[i] = threadIdx.x + i;
    float b = 1.0001f, c = 0.9999f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (OP == 0) MB_OP16("v_add_f32", "");
            if (OP == 1) MB_OP16("v_min_f32", "");
            if (OP == 2) MB_OP16("v_min3_f32", ", %17");
            if (OP == 3) MB_OP16("v_lshlrev_b32_sdwa", MB_SDWA);
            if (OP == 4) MB_OP16("v_and_b32", "");
            if (OP == 5) MB_OP16("v_lshrrev_b32", "");
            if (OP == 6) MB_OP16("v_fma_f32", ", %17");
        }
    }
    float s = 0;
    for (int i = 0; i < 16; ++i) s += a[i];
    if (s == 12345.678f) out[threadIdx.x] = s;
}

// ---------------------------------------------------------------------------------------------
// The instruction mix of the M = 4 half-plane scan (per code and lane: 4 unpacks, 8 ds_read_b128 in
// pairs, 24 adds, 4 min3, compare, select; R codes per lane-slot, reads of 3 steps in flight,
// conflict-free addresses), SWITCH = 0: nothing else; 1: two barriers per tile; 2: two barriers
// and the 128 KB tile rewritten from registers between them.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float mb_min3(float a, float b, float c)
{
    float r;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

template <int R, int SWITCH>
__global__ __launch_bounds__(512) void scan_mix_kernel(int tiles, float* out, int salt)
{
    constexpr int DEPTH = 3;
    __shared__ float4 lds[LDS_BYTES / 16];
    for (int i = threadIdx.x; i < LDS_BYTES / 16; i += 512) lds[i] = make_float4(1e-3f * (i & 255), 1.f, 2.f, 3.f);
    __syncthreads();
    const char* tb = reinterpret_cast<const char*>(lds);
    const int tid = threadIdx.x, q = tid & 3, c = tid >> 2;
    // slots {0,3,5,6} / {1,2,4,7} of a block of 8 are served together: give them the residues 0..3
    const int s8 = c & 7;
    const uint32_t res = (s8 == 0 || s8 == 1) ? 0 : (s8 == 3 || s8 == 2) ? 1 : (s8 == 5 || s8 == 4) ? 2 : 3;
    uint32_t pa[R], pb[R];
    float best[R];
    int tix[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t h = hash32((c * R + r) * 2654435761u + salt);
        const uint32_t x0 = (h & 0xfc) | res, x1 = ((h >> 8) & 0xfc) | res, x2 = ((h >> 16) & 0xfc) | res,
                       x3 = ((h >> 24) & 0xfc) | res;
        pa[r] = (x0 * 64 + q * 16) | ((x2 * 64 + q * 16 + 65536u) << 15);
        pb[r] = (x1 * 64 + q * 16) | ((x3 * 64 + q * 16 + 65536u) << 15);
        best[r] = 1e30f;
        tix[r] = -1;
    }
    struct Pair { float4 a, b; };
    auto issue = [&](int step) -> Pair {
        const int r = step / 4, m = step % 4;
        const uint32_t src = (m == 0 || m == 2) ? pa[r] : pb[r];
        uint32_t ad;
        if (m < 2) asm volatile("v_and_b32 %0, %1, %2" : "=v"(ad) : "s"(0x7fffu), "v"(src));
        else asm volatile("v_lshrrev_b32 %0, 15, %1" : "=v"(ad) : "v"(src));
        const uint32_t po = (m & 1) ? 32768 : 0;
        Pair p;
        p.a = *reinterpret_cast<const float4*>(tb + ad + po);
        p.b = *reinterpret_cast<const float4*>(tb + ad + po + 16384);
        return p;
    };
    float4 fill[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) fill[i] = make_float4(1e-3f * ((tid + i) & 255), 1.f, 2.f, 3.f);
    for (int t = 0; t < tiles; ++t) {
        if (SWITCH) {
            __syncthreads();
            if (SWITCH == 2) {
#pragma unroll
                for (int i = 0; i < 16; ++i) lds[i * 512 + tid] = fill[i];
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(fill[i].x));
        }
        Pair ring[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) ring[d] = issue(d);
        float4 sa, sb;
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const int step = 4 * r + m;
                const Pair cur = ring[step % DEPTH];
                if (step + DEPTH < 4 * R) ring[step % DEPTH] = issue(step + DEPTH);
                if (m == 0) {
                    sa = cur.a;
                    sb = cur.b;
                } else {
                    sa.x += cur.a.x; sa.y += cur.a.y; sa.z += cur.a.z; sa.w += cur.a.w;
                    sb.x += cur.b.x; sb.y += cur.b.y; sb.z += cur.b.z; sb.w += cur.b.w;
                }
                if (m == 3) {
                    float m8 = mb_min3(sa.x, sa.y, sa.z);
                    m8 = mb_min3(m8, sa.w, sb.x);
                    m8 = mb_min3(m8, sb.y, sb.z);
                    const float nb = mb_min3(m8, sb.w, best[r]);
                    tix[r] = (nb < best[r]) ? t : tix[r];
                    best[r] = nb;
                }
            }
        }
    }
    float s = 0;
    int ti = 0;
    for (int r = 0; r < R; ++r) { s += best[r]; ti += tix[r]; }
    if (s == 12345.678f) out[tid] = s + ti;
}

// streaming copy of float4 elements (HBM read + write)
__global__ __launch_bounds__(256) void copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

template <typename F>
int timed(F launch, float* ms_out)
{
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
    int rc = 0;
    for (int pass = 0; pass < 3 && rc == 0; ++pass) {          // two warm-up passes: the first launches run slower
        if (hipEventRecord(e0, 0) != hipSuccess) rc = 1;
        for (int i = 0; i < 3; ++i) launch();
        if (hipEventRecord(e1, 0) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) rc = 1;
        float ms = 0.f;
        if (rc == 0 && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = 1;
        *ms_out = ms / 3.f;
    }
    if (hipGetLastError() != hipSuccess) rc = 1;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    return rc;
}

}  // namespace

extern "C" {

// Runs microbenchmark `what` on the current device (one workgroup per compute unit) and returns the time of one
// launch in milliseconds and the work of one launch per compute unit in `units` (bytes for the LDS tests,
// wave-instructions per SIMD for the VALU tests, wave-reads of 16 bytes per lane for the scan mix).
//   0..2  ds_read_b128 / b64 / b32, lane-consecutive rows
//   3, 5, 6, 7  ds_read_b128 with 4 / 8 / 2 / 1 lanes per row of 64 / 128 / 32 / 16 bytes, rows at random positions
//   4     ds_write_b128, 128 KB per iteration
//   10..16 VALU: v_add_f32, v_min_f32, v_min3_f32, v_lshlrev_b32 (SDWA), v_and_b32, v_lshrrev_b32, v_fma_f32
//   20..22 scan mix, 31 codes per lane-slot: alone / two barriers per tile / barriers and 128 KB written per tile
//   30    streaming copy of 1 GiB (units: bytes read + written per compute unit)
// Returns 0, or 1 on an unknown test or a HIP error.  Allocates and frees a small device buffer.
int pqkm_microbench(int what, float* ms_out, double* units_out)
{
    if (!ms_out || !units_out) return 1;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return 1;
    float* out = nullptr;
    if (hipMalloc(&out, 1 << 16) != hipSuccess) return 1;
    const int it_lds = 16000, it_valu = 20000, tiles = 400;
    int rc = 1;
    switch (what) {
        case 0:
            rc = timed([&] { hipLaunchKernelGGL((lds_read_kernel<16, 64>), dim3(cus), dim3(512), 0, 0, it_lds, out, 17); }, ms_out);
            *units_out = 512.0 * 8 * 16 * it_lds;
            break;
        case 1:
            rc = timed([&] { hipLaunchKernelGGL((lds_read_kernel<8, 64>), dim3(cus), dim3(512), 0, 0, it_lds, out, 17); }, ms_out);
            *units_out = 512.0 * 8 * 8 * it_lds;
            break;
        case 2:
            rc = timed([&] { hipLaunchKernelGGL((lds_read_kernel<4, 64>), dim3(cus), dim3(512), 0, 0, it_lds, out, 17); }, ms_out);
            *units_out = 512.0 * 8 * 4 * it_lds;
            break;
        case 3:
            rc = timed([&] { hipLaunchKernelGGL((lds_read_kernel<16, 4>), dim3(cus), dim3(512), 0, 0, it_lds, out, 17); }, ms_out);
            *units_out = 512.0 * 8 * 16 * it_lds;
            break;
        case 5:
            rc = timed([&] { hipLaunchKernelGGL((lds_read_kernel<16, 8>), dim3(cus), dim3(512), 0, 0, it_lds, out, 17); }, ms_out);
            *units_out = 512.0 * 8 * 16 * it_lds;
            break;
        case 6:
            rc = timed([&] { hipLaunchKernelGGL((lds_read_kernel<16, 2>), dim3(cus), dim3(512), 0, 0, it_lds, out, 17); }, ms_out);
            *units_out = 512.0 * 8 * 16 * it_lds;
            break;
        case 7:
            rc = timed([&] { hipLaunchKernelGGL((lds_read_kernel<16, 1>), dim3(cus), dim3(512), 0, 0, it_lds, out, 17); }, ms_out);
            *units_out = 512.0 * 8 * 16 * it_lds;
            break;
        case 4:
            rc = timed([&] { hipLaunchKernelGGL(lds_write_kernel, dim3(cus), dim3(512), 0, 0, 2000, out); }, ms_out);
            *units_out = (double)LDS_BYTES * 2000;
            break;
#define MB_VALU(N, OP)                                                                                             \
    case N:                                                                                                        \
        rc = timed([&] { hipLaunchKernelGGL((valu_kernel<OP>), dim3(cus), dim3(1024), 0, 0, it_valu, out); }, ms_out); \
        *units_out = 4.0 * 64 * it_valu;                                                                           \
        break;
        MB_VALU(10, 0) MB_VALU(11, 1) MB_VALU(12, 2) MB_VALU(13, 3) MB_VALU(14, 4) MB_VALU(15, 5) MB_VALU(16, 6)
#undef MB_VALU
        case 20:
            rc = timed([&] { hipLaunchKernelGGL((scan_mix_kernel<31, 0>), dim3(cus), dim3(512), 0, 0, tiles, out, 17); }, ms_out);
            *units_out = 8.0 * 31 * 8 * tiles;
            break;
        case 21:
            rc = timed([&] { hipLaunchKernelGGL((scan_mix_kernel<31, 1>), dim3(cus), dim3(512), 0, 0, tiles, out, 17); }, ms_out);
            *units_out = 8.0 * 31 * 8 * tiles;
            break;
        case 22:
            rc = timed([&] { hipLaunchKernelGGL((scan_mix_kernel<31, 2>), dim3(cus), dim3(512), 0, 0, tiles, out, 17); }, ms_out);
            *units_out = 8.0 * 31 * 8 * tiles;
            break;
        case 30: {
            const size_t bytes = (size_t)1 << 30;
            float4 *src = nullptr, *dst = nullptr;
            if (hipMalloc(&src, bytes) == hipSuccess && hipMalloc(&dst, bytes) == hipSuccess &&
                hipMemset(src, 0, bytes) == hipSuccess) {
                rc = timed([&] { hipLaunchKernelGGL(copy_kernel, dim3(cus * 32), dim3(256), 0, 0, src, dst, bytes / 16); }, ms_out);
                *units_out = 2.0 * (double)bytes / cus;
            }
            hipFree(src);
            hipFree(dst);
            break;
        }
        default: rc = 1;
    }
    hipFree(out);
    return rc;
}

}  // extern "C"
