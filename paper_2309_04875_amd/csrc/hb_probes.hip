// Measurement aids for bench.py, built as a library of their own (libhb_probes.so).  Nothing here belongs to the
// reduced-ring ReLU interface and libhb.so does not contain or need it; the entry points allocate small device
// buffers and synchronise, which the library's own entry points never do.
//
//   hbp_clock_probe    the shader clock the GPU sustains while other work runs (one wavefront timing itself)
//   hbp_issue_probe    issue cost, in SIMD cycles per wave64 instruction, of vector-ALU instruction streams on all
//                      compute units: one instruction class alone, and two classes in runs of given lengths
//   hbp_issue_load     the same streams enqueued without waiting (a steady load to read the socket power under)
//   hbp_stream_copy    a 2-in / 2-out int64 streaming kernel (32 B per element): the memory-side ceiling for the
//                      ReLU kernels' traffic pattern, with / without the non-temporal hint and with two block orders
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdio>

#define HBP_API extern "C" __attribute__((visibility("default")))

namespace {

constexpr int kCUs = 256;       // MI355X

// ---- instruction classes ---------------------------------------------------------------------------------------
enum Op {
    kXor, kAdd, kAnd, kShr32, kCndmask,                    // two-operand 32-bit
    kBitop3, kAdd3, kAlignbit,                             // three-operand 32-bit
    kMulLo, kMulHi, kMad64,                                // multiplier
    kShr64, kLshlAdd64,                                    // 64-bit
    kSubCo, kSubbCo, kCmp,                                 // carry out, carry in and out, compare into vcc
    kCndmaskSgpr, kXorSgpr, kMulLoSgpr, kMad64Sgpr,        // a scalar-register operand
    kOps
};

const char *const kOpName[kOps] = {"v_xor_b32", "v_add_u32", "v_and_b32", "v_lshrrev_b32", "v_cndmask_b32",
                                   "v_bitop3_b32", "v_add3_u32", "v_alignbit_b32", "v_mul_lo_u32", "v_mul_hi_u32",
                                   "v_mad_u64_u32", "v_lshrrev_b64", "v_lshl_add_u64", "v_sub_co_u32 (writes vcc)",
                                   "v_subb_co_u32 (reads and writes vcc)", "v_cmp_lt_u32 (writes vcc)",
                                   "v_cndmask_b32, mask in a scalar pair", "v_xor_b32, scalar operand",
                                   "v_mul_lo_u32, scalar operand", "v_mad_u64_u32, scalar operand"};

template <int OP>
__device__ __forceinline__ void emit(uint32_t &a, uint64_t &q, uint32_t c, uint32_t cs, uint64_t ms)
{
    if constexpr (OP == kXor) asm volatile("v_xor_b32 %0, %0, %1" : "+v"(a) : "v"(c));
    if constexpr (OP == kAdd) asm volatile("v_add_u32 %0, %0, %1" : "+v"(a) : "v"(c));
    if constexpr (OP == kAnd) asm volatile("v_and_b32 %0, %0, %1" : "+v"(a) : "v"(c));
    if constexpr (OP == kShr32) asm volatile("v_lshrrev_b32 %0, 3, %0" : "+v"(a));
    if constexpr (OP == kCndmask) asm volatile("v_cndmask_b32 %0, %0, %1, vcc" : "+v"(a) : "v"(c));
    if constexpr (OP == kBitop3) asm volatile("v_bitop3_b32 %0, %0, %1, %1 bitop3:0x96" : "+v"(a) : "v"(c));
    if constexpr (OP == kAdd3) asm volatile("v_add3_u32 %0, %0, %1, %1" : "+v"(a) : "v"(c));
    if constexpr (OP == kAlignbit) asm volatile("v_alignbit_b32 %0, %0, %1, 30" : "+v"(a) : "v"(c));
    if constexpr (OP == kMulLo) asm volatile("v_mul_lo_u32 %0, %0, %1" : "+v"(a) : "v"(c));
    if constexpr (OP == kMulHi) asm volatile("v_mul_hi_u32 %0, %0, %1" : "+v"(a) : "v"(c));
    if constexpr (OP == kMad64) asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, %0" : "+v"(q) : "v"(a), "v"(c) : "vcc");
    if constexpr (OP == kShr64) asm volatile("v_lshrrev_b64 %0, 27, %0" : "+v"(q));
    if constexpr (OP == kLshlAdd64) asm volatile("v_lshl_add_u64 %0, %0, 0, %1" : "+v"(q) : "v"(q));
    if constexpr (OP == kSubCo) asm volatile("v_sub_co_u32 %0, vcc, %0, %1" : "+v"(a) : "v"(c) : "vcc");
    if constexpr (OP == kSubbCo) asm volatile("v_subb_co_u32 %0, vcc, %0, %1, vcc" : "+v"(a) : "v"(c) : "vcc");
    if constexpr (OP == kCmp) asm volatile("v_cmp_lt_u32 vcc, %0, %1" : : "v"(a), "v"(c) : "vcc");
    // cs, ms: wave-uniform values, held in scalar registers
    if constexpr (OP == kCndmaskSgpr) asm volatile("v_cndmask_b32 %0, %0, %1, %2" : "+v"(a) : "v"(c), "s"(ms));
    if constexpr (OP == kXorSgpr) asm volatile("v_xor_b32 %0, %1, %0" : "+v"(a) : "s"(cs));
    if constexpr (OP == kMulLoSgpr) asm volatile("v_mul_lo_u32 %0, %0, %1" : "+v"(a) : "s"(cs));
    if constexpr (OP == kMad64Sgpr) asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, %0" : "+v"(q) : "v"(a), "s"(cs) : "vcc");
}

// Per iteration: NA instructions of class OPA, then NB of class OPB, each class on eight independent registers.
// WAVES: wavefronts per workgroup (4 = one per SIMD; 16 = four per SIMD in one workgroup).  SYNC: a workgroup
// barrier after each run, which keeps the wavefronts that share a SIMD in the same run (bounded: every wavefront
// executes the same `iters` iterations, so every barrier is reached by all of them).
template <int OPA, int NA, int OPB, int NB, int WAVES, bool SYNC>
__global__ void __launch_bounds__(64 * WAVES) issue_kernel(uint32_t *out, int iters, long long *stamps)
{
    uint32_t a[8], b[8];
    uint64_t qa[8], qb[8];
    for (int i = 0; i < 8; ++i) {
        a[i] = threadIdx.x * 2654435761u + i;
        b[i] = blockIdx.x * 40503u + i * 7 + 1;
        qa[i] = ((uint64_t)threadIdx.x << 32) | (uint32_t)(i * 977 + blockIdx.x);
        qb[i] = ((uint64_t)blockIdx.x << 32) | (uint32_t)(i * 31 + threadIdx.x);
    }
    const uint32_t c = (0x9E3779B9u ^ threadIdx.x) | 1;
    const uint32_t cs = __builtin_amdgcn_readfirstlane(c);
    const uint64_t ms = ((uint64_t)cs << 32) | (cs * 2654435761u);
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < NA; ++i) emit<OPA>(a[i % 8], qa[i % 8], c, cs, ms);
        if (SYNC) __syncthreads();
#pragma unroll
        for (int i = 0; i < NB; ++i) emit<OPB>(b[i % 8], qb[i % 8], c, cs, ms);
        if (SYNC && NB > 0) __syncthreads();
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    uint32_t s = 0;
    for (int i = 0; i < 8; ++i) s ^= a[i] ^ b[i] ^ (uint32_t)qa[i] ^ (uint32_t)(qa[i] >> 32) ^ (uint32_t)qb[i] ^ (uint32_t)(qb[i] >> 32);
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (threadIdx.x == 0 && blockIdx.x < 8) {
        stamps[2 * blockIdx.x] = c1 - c0;
        stamps[2 * blockIdx.x + 1] = w1 - w0;
    }
}

struct Probe {
    const char *name;
    int per_iteration;                 // instructions per iteration per wavefront
    int waves_per_block;
    void (*launch)(int blocks, uint32_t *out, int iters, long long *stamps, hipStream_t stream);
};

template <int OPA, int NA, int OPB, int NB, int WAVES, bool SYNC>
void launch_issue(int blocks, uint32_t *out, int iters, long long *stamps, hipStream_t stream)
{
    hipLaunchKernelGGL((issue_kernel<OPA, NA, OPB, NB, WAVES, SYNC>), dim3(blocks), dim3(64 * WAVES), 0, stream, out, iters, stamps);
}

#define ALONE(OP) {nullptr, 64, 4, &launch_issue<OP, 64, kXor, 0, 4, false>}
#define RUNS(NAME, OPA, NA, OPB, NB) {NAME, (NA) + (NB), 4, &launch_issue<OPA, NA, OPB, NB, 4, false>}
#define RUNS16(NAME, OPA, NA, OPB, NB, SYNC) {NAME, (NA) + (NB), 16, &launch_issue<OPA, NA, OPB, NB, 16, SYNC>}

// The first kOps entries are the classes alone, in enum order (their names come from kOpName).
const Probe kProbes[] = {
    ALONE(kXor), ALONE(kAdd), ALONE(kAnd), ALONE(kShr32), ALONE(kCndmask), ALONE(kBitop3), ALONE(kAdd3), ALONE(kAlignbit),
    ALONE(kMulLo), ALONE(kMulHi), ALONE(kMad64), ALONE(kShr64), ALONE(kLshlAdd64),
    ALONE(kSubCo), ALONE(kSubbCo), ALONE(kCmp), ALONE(kCndmaskSgpr), ALONE(kXorSgpr), ALONE(kMulLoSgpr), ALONE(kMad64Sgpr),
    RUNS("xor x1 / mul_lo x1", kXor, 1, kMulLo, 1),
    RUNS("xor x2 / mul_lo x2", kXor, 2, kMulLo, 2),
    RUNS("xor x8 / mul_lo x8", kXor, 8, kMulLo, 8),
    RUNS("xor x64 / mul_lo x64", kXor, 64, kMulLo, 64),
    RUNS("xor x128 / mul_lo x128", kXor, 128, kMulLo, 128),
    RUNS("xor x3 / mul_lo x1", kXor, 3, kMulLo, 1),
    RUNS("xor x1 / mul_lo x3", kXor, 1, kMulLo, 3),
    RUNS("xor x8 / bitop3 x8", kXor, 8, kBitop3, 8),
    RUNS("xor x8 / lshrrev_b64 x8", kXor, 8, kShr64, 8),
    RUNS("xor x8 / add3 x8", kXor, 8, kAdd3, 8),
    RUNS("xor x8 / and x8", kXor, 8, kAnd, 8),
    RUNS("mul_lo x8 / mad_u64_u32 x8", kMulLo, 8, kMad64, 8),
    RUNS("cmp x1 / cndmask(vcc) x1", kCmp, 1, kCndmask, 1),
    RUNS("sub_co x1 / subb_co x1 (64-bit subtract)", kSubCo, 1, kSubbCo, 1),
    RUNS16("16-wave groups: xor x128 alone", kXor, 128, kMulLo, 0, false),
    RUNS16("16-wave groups: mul_lo x128 alone", kMulLo, 128, kXor, 0, false),
    RUNS16("16-wave groups: xor x128 / mul_lo x128, free-running", kXor, 128, kMulLo, 128, false),
    RUNS16("16-wave groups: xor x128 / mul_lo x128, barrier after each run", kXor, 128, kMulLo, 128, true),
    RUNS16("16-wave groups: xor x32 / mul_lo x32, free-running", kXor, 32, kMulLo, 32, false),
    RUNS16("16-wave groups: xor x32 / mul_lo x32, barrier after each run", kXor, 32, kMulLo, 32, true),
};
constexpr int kProbeCount = (int)(sizeof(kProbes) / sizeof(kProbes[0]));

uint32_t *g_out = nullptr;
long long *g_stamps = nullptr;

hipError_t scratch_buffers()
{
    if (g_out != nullptr) return hipSuccess;
    hipError_t e = hipMalloc(&g_out, (size_t)kCUs * 8 * 1024 * sizeof(uint32_t));
    if (e != hipSuccess) return e;
    e = hipMalloc(&g_stamps, 16 * sizeof(long long));
    if (e != hipSuccess) return e;
    return hipMemset(g_stamps, 0, 16 * sizeof(long long));
}

__global__ void __launch_bounds__(64) clock_probe_kernel(uint64_t spins, uint64_t *stamps)
{
    uint64_t z = threadIdx.x;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (uint64_t i = 0; i < spins; ++i) {      // a dependent chain: multiply, xor-shift
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull + i;
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    if (threadIdx.x == 0) {
        stamps[0] = (uint64_t)(c1 - c0) + (z == 0x5bd1e995u ? 1 : 0);   // keeps the loop alive
        stamps[1] = (uint64_t)(w1 - w0);
    }
}

// ---- 2-in / 2-out streaming ------------------------------------------------------------------------------------
typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));
constexpr int kChunks = 4;      // 16-byte accesses per lane and array

// MAP 0: block b takes consecutive wave-chunks (blocks resident together stream neighbouring addresses);
// MAP 1: blocks b, b + 8, b + 16, ... (one XCD under round-robin dispatch) take a contiguous eighth of the arrays.
template <bool NT, int MAP>
__global__ void __launch_bounds__(256) stream_kernel(const u64x2 *x0, const u64x2 *x1, u64x2 *o0, u64x2 *o1, uint64_t pairs)
{
    uint64_t blk = blockIdx.x;
    if (MAP == 1) {
        const uint64_t per = gridDim.x / 8;
        if (blk < per * 8) blk = (blk % 8) * per + blk / 8;
    }
    const uint64_t wave = (blk * 256 + threadIdx.x) / 64;
    const uint64_t base = wave * (64 * kChunks) + threadIdx.x % 64;
    u64x2 a[kChunks], b[kChunks];
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
        const uint64_t i = base + c * 64;
        if (i < pairs) {
            a[c] = NT ? __builtin_nontemporal_load(&x0[i]) : x0[i];
            b[c] = NT ? __builtin_nontemporal_load(&x1[i]) : x1[i];
        }
    }
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
        const uint64_t i = base + c * 64;
        if (i < pairs) {
            const u64x2 r0 = a[c] + b[c], r1 = a[c] ^ b[c];
            if (NT) {
                __builtin_nontemporal_store(r0, &o0[i]);
                __builtin_nontemporal_store(r1, &o1[i]);
            } else {
                o0[i] = r0;
                o1[i] = r1;
            }
        }
    }
}

}  // namespace

HBP_API int hbp_issue_probe_count(void) { return kProbeCount; }
HBP_API int hbp_issue_class_count(void) { return kOps; }

HBP_API const char *hbp_issue_probe_name(int index)
{
    if (index < 0 || index >= kProbeCount) return "";
    return kProbes[index].name ? kProbes[index].name : kOpName[index];
}

// Enqueue `launches` launches of probe `index` at `waves_per_simd` on `stream` without waiting.
// Returns 0, or a HIP error code.
HBP_API int hbp_issue_load(int index, int waves_per_simd, int iters, int launches, void *stream)
{
    if (index < 0 || index >= kProbeCount || waves_per_simd < 1 || waves_per_simd > 8 || iters < 1) return -1;
    const Probe &p = kProbes[index];
    const int per_block = p.waves_per_block / 4;                // wavefronts per SIMD that one workgroup brings
    if (waves_per_simd % per_block != 0) return -1;
    hipError_t e = scratch_buffers();
    if (e != hipSuccess) return (int)e;
    const int blocks = kCUs * (waves_per_simd / per_block);
    for (int i = 0; i < launches; ++i) p.launch(blocks, g_out, iters, g_stamps, (hipStream_t)stream);
    return (int)hipGetLastError();
}

// Runs probe `index` (warm-up launch, then one timed launch) and waits.  result (HOST, 4 doubles): duration in ms,
// shader clock in MHz measured inside the timed launch, SIMD cycles per wave64 instruction, instructions per
// wavefront of the timed launch.
HBP_API int hbp_issue_probe(int index, int waves_per_simd, int iters, double *result)
{
    if (result == nullptr) return -1;
    int st = hbp_issue_load(index, waves_per_simd, iters, 2, nullptr);      // warm the clocks
    if (st != 0) return st;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -2;
    hipError_t e = hipEventRecord(e0, nullptr);
    st = hbp_issue_load(index, waves_per_simd, iters, 1, nullptr);
    if (e == hipSuccess) e = hipEventRecord(e1, nullptr);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != 0 || e != hipSuccess) return st != 0 ? st : (int)e;
    long long h[16];
    if (hipMemcpy(h, g_stamps, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return -2;
    double ticks = 0, wall = 0;
    for (int i = 0; i < 8; ++i) {
        ticks += (double)h[2 * i];
        wall += (double)h[2 * i + 1];
    }
    const double mhz = wall > 0 ? 100.0 * ticks / wall : 0.0;               // the wall clock counts at 100 MHz
    const Probe &p = kProbes[index];
    const double per_wave = (double)iters * p.per_iteration;
    const double per_simd = per_wave * waves_per_simd;
    result[0] = ms;
    result[1] = mhz;
    result[2] = ms * 1e-3 * mhz * 1e6 / per_simd;
    result[3] = per_wave;
    return 0;
}

// One wavefront reads the shader-clock counter and the constant 100 MHz counter around `spins` iterations of a
// dependent arithmetic chain (bounded: exactly `spins` iterations, at most 2^24).  stamps: DEVICE, 2 uint64:
// {shader-clock ticks, 100 MHz ticks}; MHz = 100 * stamps[0] / stamps[1].  Enqueued on `stream`, no waiting.
HBP_API int hbp_clock_probe(uint64_t spins, uint64_t *stamps, void *stream)
{
    if (stamps == nullptr || spins == 0 || spins > (1ull << 24) || ((uintptr_t)stamps & 7u) != 0) return -1;
    hipLaunchKernelGGL(clock_probe_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, spins, stamps);
    return (int)hipGetLastError();
}

// out0 = x0 + x1, out1 = x0 ^ x1 over n int64 elements (n even, 16-byte aligned DEVICE buffers); enqueued, no waiting.
HBP_API int hbp_stream_copy(int nontemporal, int xcd_contiguous, const uint64_t *x0, const uint64_t *x1, uint64_t *o0,
                            uint64_t *o1, uint64_t n, void *stream)
{
    if (n == 0 || n % 2 != 0 || !x0 || !x1 || !o0 || !o1) return -1;
    if ((((uintptr_t)x0 | (uintptr_t)x1 | (uintptr_t)o0 | (uintptr_t)o1) & 15u) != 0) return -1;
    const uint64_t pairs = n / 2;
    const uint64_t waves = (pairs + 64 * kChunks - 1) / (64 * kChunks);
    const uint64_t blocks = (waves + 3) / 4;
    if (blocks > 0x7fffffffull) return -1;
    const dim3 grid((unsigned)blocks), blk(256);
    const u64x2 *a = (const u64x2 *)x0, *b = (const u64x2 *)x1;
    u64x2 *c = (u64x2 *)o0, *d = (u64x2 *)o1;
    hipStream_t q = (hipStream_t)stream;
    if (nontemporal && xcd_contiguous) hipLaunchKernelGGL((stream_kernel<true, 1>), grid, blk, 0, q, a, b, c, d, pairs);
    else if (nontemporal) hipLaunchKernelGGL((stream_kernel<true, 0>), grid, blk, 0, q, a, b, c, d, pairs);
    else if (xcd_contiguous) hipLaunchKernelGGL((stream_kernel<false, 1>), grid, blk, 0, q, a, b, c, d, pairs);
    else hipLaunchKernelGGL((stream_kernel<false, 0>), grid, blk, 0, q, a, b, c, d, pairs);
    return (int)hipGetLastError();
}
