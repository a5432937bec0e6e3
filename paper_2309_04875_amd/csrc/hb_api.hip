// C ABI of the library (include/hb.h): argument checks on the host, closed-form opened-bit counts,
// kernel selection by slice width, launch on the caller's stream.  No allocation, no synchronisation.
#include "../../include/hb.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <utility>
#include <vector>

#include "hb_eco.hpp"
#include "hb_float.hpp"
#include "hb_kernels.hpp"
#include "hb_launch.hpp"
#include "hb_multiparty.hpp"
#include "hb_party.hpp"

namespace {

thread_local char g_hip_error[256] = "";

int fail_hip(hipError_t e, const char *what)
{
    std::snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
    (void)hipGetLastError();
    return HB_EHIP;
}

bool valid_slice(int k, int m) { return k >= 0 && m > k && m <= 64; }

int rounds_of(int w) { return hb::ceil_log2(w); }

struct Range {
    uintptr_t lo, hi;
};

Range range_of(const void *p, size_t n) { return Range{(uintptr_t)p, (uintptr_t)p + n * sizeof(int64_t)}; }

bool same(Range a, Range b) { return a.lo == b.lo; }
bool disjoint(Range a, Range b) { return a.hi <= b.lo || b.hi <= a.lo; }

// The buffer must be memory the GPU can address, and [p, p + 8n) must lie inside one allocation.
int check_device_bytes(const void *p, size_t bytes);

int check_device_buffer(const void *p, size_t n) { return check_device_bytes(p, n * sizeof(int64_t)); }

int check_device_bytes(const void *p, size_t bytes)
{
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return HB_EINVAL;  // not known to the HIP runtime: plain host memory or a wild pointer
    }
    switch (attr.type) {
    case hipMemoryTypeDevice: {   // memory of another GPU is not addressable from the kernels launched here
        int current = -1;
        if (hipGetDevice(&current) != hipSuccess || attr.device != current) {
            (void)hipGetLastError();
            return HB_EINVAL;
        }
        break;
    }
    case hipMemoryTypeManaged:
        break;
    case hipMemoryTypeHost:  // pinned host memory is usable only through its device-side address
        if (attr.devicePointer != p) return HB_EINVAL;
        break;
    default:  // unregistered host memory, arrays
        return HB_EINVAL;
    }
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    e = hipMemGetAddressRange(&base, &size, (hipDeviceptr_t)p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return HB_OK;  // allocation kinds without a queryable range: the attribute check has passed
    }
    const uintptr_t lo = (uintptr_t)base, hi = lo + size;
    const Range r{(uintptr_t)p, (uintptr_t)p + bytes};
    return (r.lo >= lo && r.hi <= hi) ? HB_OK : HB_EINVAL;
}

int check_common(const void *const *ptrs, int count, size_t n)
{
    if (n > HB_MAX_ELEMENTS) return HB_EINVAL;
    if (n == 0) return HB_OK;
    for (int i = 0; i < count; ++i) {
        if (ptrs[i] == nullptr) return HB_EINVAL;
    }
    for (int i = 0; i < count; ++i) {
        if (((uintptr_t)ptrs[i] & 7u) != 0) return HB_EALIGN;
    }
    for (int i = 0; i < count; ++i) {
        const int st = check_device_buffer(ptrs[i], n);
        if (st != HB_OK) return st;
    }
    return HB_OK;
}

// A device buffer of n floats with the given alignment.
int check_float_buffer(const void *p, size_t n, unsigned align)
{
    if (p == nullptr) return HB_EINVAL;
    if (((uintptr_t)p & (align - 1)) != 0) return HB_EALIGN;
    return check_device_bytes(p, n * sizeof(float));
}

bool all_aligned16(const void *const *ptrs, int count)
{
    for (int i = 0; i < count; ++i) {
        if (((uintptr_t)ptrs[i] & 15u) != 0) return false;
    }
    return true;
}

// Argument rules of one tensor of a call (no launch): slice, pointers, alignment, device memory, overlaps.
int validate_tensor(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, const int64_t *out0,
                    const int64_t *out1)
{
    if (!valid_slice(k, m)) return HB_EINVAL;
    const void *ptrs[4] = {share0, share1, out0, out1};
    const int st = check_common(ptrs, 4, n);
    if (st != HB_OK) return st;
    if (n > 0) {
        const Range i0 = range_of(share0, n), i1 = range_of(share1, n), r0 = range_of(out0, n), r1 = range_of(out1, n);
        // an output may coincide with an input; every other overlap is refused
        if (!disjoint(r0, r1)) return HB_EINVAL;
        if (!(same(r0, i0) || disjoint(r0, i0)) || !(same(r0, i1) || disjoint(r0, i1))) return HB_EINVAL;
        if (!(same(r1, i0) || disjoint(r1, i0)) || !(same(r1, i1) || disjoint(r1, i1))) return HB_EINVAL;
    }
    return HB_OK;
}

uint64_t mode_bits(int mode, int k, int m, size_t n)
{
    return hb_opened_bits_ex(hb::op_of(mode) == hb::kRelu, k, m, n,
                             hb::shared_of(mode) ? HB_DEALER_SHARED_MASK : HB_DEALER_PER_GATE);
}

// mode of an operation (kDrelu or kRelu) on a dealer layout; -1 for an unknown layout
int mode_on(int op, int dealer)
{
    if (dealer == HB_DEALER_PER_GATE) return op;
    if (dealer == HB_DEALER_SHARED_MASK) return op + hb::kDreluShared;
    return -1;
}

// One kernel launch, ready to be enqueued: either a set of tensors of one width on wave-tiles (large or small) or one
// tensor on the thread-per-group kernel.
struct LaunchItem {
    hb::BatchLauncher tiles = nullptr;   // wave-tile launch of args.t[0 .. args.count)
    hb::GroupLauncher single = nullptr;  // per-tensor launch of args.t[0]
    hb::BatchArgs args = {};
    bool vec16 = false;
};

hipError_t enqueue(const LaunchItem &it, hipStream_t stream)
{
    if (it.tiles != nullptr) return it.tiles(it.args, stream);
    const hb::BatchTensor &d = it.args.t[0];
    return it.single(d.x0, d.x1, d.n, d.k, d.seedB, d.seedA, d.o0, d.o1, it.vec16, stream);
}

// Launches with fewer large wave-tiles than this take the small wave-tile kernels (where the width has them): below
// about one wavefront per SIMD a launch lasts as long as one wavefront's instruction stream, which they shorten.
// HB_SMALL_TILE_LIMIT in the environment (read once) overrides the limit; 0 switches the small tiles off.
uint64_t small_tile_limit()
{
    static const uint64_t limit = [] {
        const char *v = std::getenv("HB_SMALL_TILE_LIMIT");
        return v != nullptr ? (uint64_t)std::strtoull(v, nullptr, 10) : (uint64_t)1536;
    }();
    return limit;
}

void fill_tensor(hb::BatchTensor &d, const hb_tensor &t)
{
    d.x0 = (const uint64_t *)t.share0;
    d.x1 = (const uint64_t *)t.share1;
    d.o0 = (uint64_t *)t.out0;
    d.o1 = (uint64_t *)t.out1;
    d.n = t.n;
    d.seedB = hb::stream_word(t.seed, 0);
    d.seedA = hb::stream_word(t.seed, 1);
    d.k = t.k;
}

// Turns validated tensors (all of `mode`) into launches: tensors of one slice width that have a wave-tile kernel
// share launches of up to kBatchMax tensors; the others get one launch each.  Tensors with n == 0 are skipped.
// Returns HB_OK or HB_EHIP (no kernel for a width: a build problem).
int plan_launches(int mode, const hb_tensor *tensors, size_t count, std::vector<LaunchItem> &items)
{
    std::vector<char> taken(count, 0);
    for (size_t i = 0; i < count; ++i) {
        if (taken[i]) continue;
        taken[i] = 1;
        const hb_tensor &first = tensors[i];
        if (first.n == 0) continue;
        const int w = first.m - first.k;
        const hb::BatchLauncher big = hb::force_group_kernel() ? nullptr : hb::launcher_table().batch[mode][w - 1];
        if (big == nullptr) {
            LaunchItem it;
            it.single = hb::launcher_table().f[mode][w - 1];
            if (it.single == nullptr) return fail_hip(hipErrorInvalidDeviceFunction, "no kernel was built for this slice width");
            fill_tensor(it.args.t[0], first);
            it.args.count = 1;
            const void *ptrs[4] = {first.share0, first.share1, first.out0, first.out1};
            it.vec16 = all_aligned16(ptrs, 4);
            items.push_back(it);
            continue;
        }
        // every tensor of this width, in order
        std::vector<size_t> same;
        for (size_t j = i; j < count; ++j) {
            if ((j == i || !taken[j]) && tensors[j].m - tensors[j].k == w && tensors[j].n > 0) {
                taken[j] = 1;
                same.push_back(j);
            }
        }
        const uint64_t per_big = (uint64_t)hb::tile_elements(w);
        uint64_t big_tiles = 0;
        for (size_t j : same) big_tiles += (tensors[j].n + per_big - 1) / per_big;
        const hb::BatchLauncher small = hb::launcher_table().small[mode][w - 1];
        const bool use_small = small != nullptr && big_tiles < small_tile_limit();
        const uint64_t per_tile = use_small ? (uint64_t)hb::small_tile_elements(w) : per_big;
        LaunchItem it;
        it.tiles = use_small ? small : big;
        for (size_t j : same) {
            if (it.args.count == hb::kBatchMax) {
                items.push_back(it);
                it.args = hb::BatchArgs{};
            }
            const hb_tensor &t = tensors[j];
            fill_tensor(it.args.t[it.args.count], t);
            it.args.tile_end[it.args.count] = (it.args.count ? it.args.tile_end[it.args.count - 1] : 0) + (t.n + per_tile - 1) / per_tile;
            ++it.args.count;
        }
        items.push_back(it);
    }
    return HB_OK;
}

int run(int mode, const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed, int64_t *out0,
        int64_t *out1, uint64_t *opened_bits, void *stream)
{
    const int st = validate_tensor(share0, share1, n, k, m, out0, out1);
    if (st != HB_OK) return st;
    const int w = m - k;
    uint64_t bits = 0;
    if (mode == hb::kSign) {
        bits = (uint64_t)n * (2ull * (uint64_t)w * (1 + 2 * (uint64_t)rounds_of(w)));
    } else {
        bits = mode_bits(mode, k, m, n);
    }
    if (n > 0) {
        const uint64_t seedB = hb::stream_word(seed, 0), seedA = hb::stream_word(seed, 1);
        const uint64_t per_big = (uint64_t)hb::tile_elements(w);
        const hb::BatchLauncher small = hb::force_group_kernel() ? nullptr : hb::launcher_table().small[mode][w - 1];
        hipError_t e;
        if (small != nullptr && (n + per_big - 1) / per_big < small_tile_limit()) {
            hb::BatchArgs args = {};
            const hb_tensor t = {share0, share1, out0, out1, n, k, m, seed};
            fill_tensor(args.t[0], t);
            const uint64_t per_tile = (uint64_t)hb::small_tile_elements(w);
            args.tile_end[0] = (n + per_tile - 1) / per_tile;
            args.count = 1;
            e = small(args, (hipStream_t)stream);
        } else {
            const void *ptrs[4] = {share0, share1, out0, out1};
            const hb::GroupLauncher f = hb::launcher_table().f[mode][w - 1];
            if (f == nullptr) return fail_hip(hipErrorInvalidDeviceFunction, "no kernel was built for this slice width");
            e = f((const uint64_t *)share0, (const uint64_t *)share1, (uint64_t)n, k, seedB, seedA, (uint64_t *)out0,
                  (uint64_t *)out1, all_aligned16(ptrs, 4), (hipStream_t)stream);
        }
        if (e != hipSuccess) return fail_hip(e, "kernel launch");
    }
    if (opened_bits) *opened_bits = bits;
    return HB_OK;
}

// DReLU / ReLU among `parties` parties.  shares / outs: host arrays of `parties` device pointers.
int run_mp(int op, const int64_t *const *shares, int parties, size_t n, int k, int m, uint64_t seed,
           int64_t *const *outs, uint64_t *opened_bits, void *stream)
{
    if (parties < 2 || parties > hb::kMaxParties) return HB_EINVAL;
    if (shares == nullptr || outs == nullptr) return HB_EINVAL;
    if (parties == 2) return run(op, shares[0], shares[1], n, k, m, seed, outs[0], outs[1], opened_bits, stream);
    if (!valid_slice(k, m)) return HB_EINVAL;
    const void *ptrs[2 * hb::kMaxParties];
    for (int q = 0; q < parties; ++q) {
        ptrs[q] = shares[q];
        ptrs[parties + q] = outs[q];
    }
    const int st = check_common(ptrs, 2 * parties, n);
    if (st != HB_OK) return st;
    if (n > 0) {
        // an output may coincide with an input; every other overlap is refused
        for (int q = 0; q < parties; ++q) {
            const Range out = range_of(outs[q], n);
            for (int t = 0; t < parties; ++t) {
                const Range in = range_of(shares[t], n);
                if (!(same(out, in) || disjoint(out, in))) return HB_EINVAL;
                if (t != q && !disjoint(out, range_of(outs[t], n))) return HB_EINVAL;
            }
        }
        hb::MpPointers ptr = {};
        for (int q = 0; q < parties; ++q) {
            ptr.x[q] = (const uint64_t *)shares[q];
            ptr.o[q] = (uint64_t *)outs[q];
        }
        const hb::MpLauncher f = hb::launcher_table().mp[parties - 3][op][m - k - 1];
        if (f == nullptr) return fail_hip(hipErrorInvalidDeviceFunction, "no kernel was built for this slice width");
        const hipError_t e = f(ptr, (uint64_t)n, k, hb::stream_word(seed, 0), hb::stream_word(seed, 1),
                               (hipStream_t)stream);
        if (e != hipSuccess) return fail_hip(e, "kernel launch");
    }
    if (opened_bits) *opened_bits = hb_opened_bits_mp(op == hb::kRelu, parties, k, m, n);
    return HB_OK;
}

// Workspace of the party-faithful path: [wire 0][wire 1][state 0][state 1], every region 256-byte aligned.
// state p = S, P, G, Z (one word per group each) and D (one word per element).
struct PartyLayout {
    uint64_t groups, wire_words, wire_off[2], state_off[2], total_bytes;
};

PartyLayout party_layout(size_t n, int k, int m, int dealer = HB_DEALER_PER_GATE)
{
    const int w = m - k;
    const uint64_t L = (64 / w) > 32 ? 32 : (uint64_t)(64 / w);
    const uint64_t R = (uint64_t)rounds_of(w);
    const uint64_t per_round = dealer == HB_DEALER_SHARED_MASK ? 3 : 4;
    PartyLayout lay = {};
    lay.groups = ((uint64_t)n + L - 1) / L;
    lay.wire_words = 2 * lay.groups + per_round * lay.groups * R + ((uint64_t)n + 63) / 64 + 2 * (uint64_t)n;
    auto up = [](uint64_t b) { return (b + 255) & ~255ull; };
    const uint64_t wire_bytes = up(8 * lay.wire_words), state_bytes = up(8 * (4 * lay.groups + (uint64_t)n));
    lay.wire_off[0] = 0;
    lay.wire_off[1] = wire_bytes;
    lay.state_off[0] = 2 * wire_bytes;
    lay.state_off[1] = 2 * wire_bytes + state_bytes;
    lay.total_bytes = 2 * wire_bytes + 2 * state_bytes;
    return lay;
}

// Argument rules of a set of tensors (no launch): each tensor's own rules, then no output of one tensor over any
// buffer of another.  bits: the opened-bit count of the set.
int validate_set(int mode, const hb_tensor *tensors, size_t count, uint64_t *bits)
{
    if (count > 0 && tensors == nullptr) return HB_EINVAL;
    if (count > 4096) return HB_EINVAL;
    for (size_t i = 0; i < count; ++i) {
        const hb_tensor &t = tensors[i];
        const int st = validate_tensor(t.share0, t.share1, t.n, t.k, t.m, t.out0, t.out1);
        if (st != HB_OK) return st;
    }
    for (size_t i = 0; i < count; ++i) {
        const hb_tensor &a = tensors[i];
        if (a.n == 0) continue;
        const Range outs[2] = {range_of(a.out0, a.n), range_of(a.out1, a.n)};
        for (size_t j = 0; j < count; ++j) {
            const hb_tensor &b = tensors[j];
            if (j == i || b.n == 0) continue;
            const Range others[4] = {range_of(b.share0, b.n), range_of(b.share1, b.n), range_of(b.out0, b.n),
                                     range_of(b.out1, b.n)};
            for (const Range &o : outs) {
                for (const Range &r : others) {
                    if (!disjoint(o, r)) return HB_EINVAL;
                }
            }
        }
    }
    uint64_t total = 0;
    for (size_t i = 0; i < count; ++i) total += mode_bits(mode, tensors[i].k, tensors[i].m, tensors[i].n);
    *bits = total;
    return HB_OK;
}

int run_batch(int mode, const hb_tensor *tensors, size_t count, uint64_t *opened_bits, void *stream)
{
    // validate everything first: on error nothing is enqueued
    uint64_t bits = 0;
    int st = validate_set(mode, tensors, count, &bits);
    if (st != HB_OK) return st;
    std::vector<LaunchItem> items;
    st = plan_launches(mode, tensors, count, items);
    if (st != HB_OK) return st;
    for (const LaunchItem &it : items) {
        const hipError_t e = enqueue(it, (hipStream_t)stream);
        if (e != hipSuccess) return fail_hip(e, "kernel launch");
    }
    if (opened_bits) *opened_bits = bits;
    return HB_OK;
}

// ---- the library's own workspace for hb_relu_party_static ---------------------------------------------------
// One array per GPU (each device that loads the code object holds its own copy at its own address, until the
// process ends).  In host code the array's name is only a handle for the symbol lookup below; kernels get the
// device address that the lookup returned, as an ordinary argument.
static __device__ __align__(256) unsigned char scratch[HB_PARTY_STATIC_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_of_device[kMaxDevices];

// Device address of `scratch` on the current device; looked up once per device, with that device current.
int party_scratch_of_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return HB_EINVAL;
    void *p = g_scratch_of_device[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr) return fail_hip(e, "hipGetSymbolAddress(scratch)");
        g_scratch_of_device[dev].store(p, std::memory_order_release);   // racing threads store the same address
    }
    *out = p;
    return HB_OK;
}

// The party-faithful path on a given workspace.  `own_workspace`: the workspace is the library's static array
// (its address and size are known good), otherwise a caller's buffer that is checked like every other argument.
int run_party(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed, int dealer,
              int64_t *out0, int64_t *out1, void *workspace, size_t workspace_bytes, bool own_workspace,
              uint64_t *wire_bytes, void *stream)
{
    if (dealer != HB_DEALER_PER_GATE && dealer != HB_DEALER_SHARED_MASK) return HB_EINVAL;
    int st = validate_tensor(share0, share1, n, k, m, out0, out1);
    if (st != HB_OK) return st;
    const PartyLayout lay = party_layout(n, k, m, dealer);
    if (n > 0) {
        if (workspace == nullptr || workspace_bytes < lay.total_bytes) return HB_EINVAL;
        if (((uintptr_t)workspace & 255u) != 0) return HB_EALIGN;
        if (!own_workspace) {
            st = check_device_buffer(workspace, (lay.total_bytes + 7) / 8);
            if (st != HB_OK) return st;
        }
        const Range ws{(uintptr_t)workspace, (uintptr_t)workspace + lay.total_bytes};
        const Range bufs[4] = {range_of(share0, n), range_of(share1, n), range_of(out0, n), range_of(out1, n)};
        for (const Range &b : bufs) {
            if (!disjoint(ws, b)) return HB_EINVAL;
        }
        // each party re-reads its share after the other party's kernels have run: no in-place operation here
        if (!disjoint(bufs[2], bufs[0]) || !disjoint(bufs[2], bufs[1]) || !disjoint(bufs[3], bufs[0]) ||
            !disjoint(bufs[3], bufs[1]))
            return HB_EINVAL;
    }
    if (wire_bytes) *wire_bytes = 8 * lay.wire_words;
    if (n == 0) return HB_OK;

    const int w = m - k;
    hb::PartyShape s = {};
    s.w = w;
    s.R = rounds_of(w);
    s.L = (64 / w) > 32 ? 32 : 64 / w;
    s.k = k;
    s.shared = dealer == HB_DEALER_SHARED_MASK;
    s.per_round = s.shared ? 3 : 4;
    s.words_per_group = (uint64_t)(s.shared ? 5 + 8 * s.R + 1 : 5 * (1 + 2 * s.R) + 1);
    s.field = (w == 64) ? ~0ull : ((1ull << w) - 1);
    auto repeat = [&](uint64_t f) {
        uint64_t r = 0;
        for (int j = 0; j < s.L; ++j) r |= f << (j * w);
        return r;
    };
    s.ones = repeat(1);
    s.live = repeat(s.field);
    for (int r = 0; r < 6; ++r) {
        const int sh = 1 << r;
        s.keep[r] = (sh >= w) ? 0 : repeat((s.field << sh) & s.field);
    }
    s.keep1 = (1 >= w) ? 0 : repeat((s.field << 1) & s.field);

    hb::PartyCtx c = {};
    char *base = (char *)workspace;
    c.x[0] = (const uint64_t *)share0;
    c.x[1] = (const uint64_t *)share1;
    c.out[0] = (uint64_t *)out0;
    c.out[1] = (uint64_t *)out1;
    c.n = n;
    c.groups = lay.groups;
    c.seedB = hb::stream_word(seed, 0);
    c.seedA = hb::stream_word(seed, 1);
    for (int p = 0; p < 2; ++p) {
        c.wire[p] = (uint64_t *)(base + lay.wire_off[p]);
        uint64_t *state = (uint64_t *)(base + lay.state_off[p]);
        c.S[p] = state;
        c.P[p] = state + lay.groups;
        c.G[p] = state + 2 * lay.groups;
        c.Z[p] = state + 3 * lay.groups;
        c.D[p] = state + 4 * lay.groups;
    }
    c.off_b2a = 2 * lay.groups + (uint64_t)s.per_round * lay.groups * (uint64_t)s.R;
    c.off_mul = c.off_b2a + (n + 63) / 64;

    auto grid_for = [](uint64_t threads) { return dim3((unsigned)((threads + hb::kPartyBlock - 1) / hb::kPartyBlock), 2); };
    if ((lay.groups + hb::kPartyBlock - 1) / hb::kPartyBlock > 0x7fffffffull || (n + hb::kPartyBlock - 1) / hb::kPartyBlock > 0x7fffffffull)
        return HB_EINVAL;
    hipStream_t q = (hipStream_t)stream;
    const dim3 blk(hb::kPartyBlock);
    hipLaunchKernelGGL(hb::party_slice_kernel, grid_for(lay.groups), blk, 0, q, c, s);
    for (int r = 0; r < s.R; ++r) hipLaunchKernelGGL(hb::party_round_kernel, grid_for(lay.groups), blk, 0, q, c, s, r);
    hipLaunchKernelGGL(hb::party_sign_kernel, grid_for(lay.groups), blk, 0, q, c, s);
    hipLaunchKernelGGL(hb::party_b2a_kernel, grid_for((n + 63) / 64), blk, 0, q, c, s);
    hipLaunchKernelGGL(hb::party_mul_send_kernel, grid_for(n), blk, 0, q, c, s);
    hipLaunchKernelGGL(hb::party_mul_finish_kernel, grid_for(n), blk, 0, q, c, s);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    return HB_OK;
}

}  // namespace

namespace hb {
LauncherTable &launcher_table()
{
    static LauncherTable table = {};
    return table;
}

bool force_group_kernel()
{
    static const bool forced = [] {
        const char *v = std::getenv("HB_KERNEL");
        return v != nullptr && std::strcmp(v, "group") == 0;
    }();
    return forced;
}
}  // namespace hb

extern "C" {

int hb_drelu(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed, int64_t *out0,
             int64_t *out1, uint64_t *opened_bits, void *stream)
{
    return run(hb::kDrelu, share0, share1, n, k, m, seed, out0, out1, opened_bits, stream);
}

int hb_relu(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed, int64_t *out0,
            int64_t *out1, uint64_t *opened_bits, void *stream)
{
    return run(hb::kRelu, share0, share1, n, k, m, seed, out0, out1, opened_bits, stream);
}

int hb_sign_shares(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed, int64_t *out0,
                   int64_t *out1, uint64_t *opened_bits, void *stream)
{
    return run(hb::kSign, share0, share1, n, k, m, seed, out0, out1, opened_bits, stream);
}

int hb_relu_batch(const hb_tensor *tensors, size_t count, uint64_t *opened_bits, void *stream)
{
    return run_batch(hb::kRelu, tensors, count, opened_bits, stream);
}

int hb_drelu_batch(const hb_tensor *tensors, size_t count, uint64_t *opened_bits, void *stream)
{
    return run_batch(hb::kDrelu, tensors, count, opened_bits, stream);
}

int hb_drelu_ex(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed, int dealer,
                int64_t *out0, int64_t *out1, uint64_t *opened_bits, void *stream)
{
    const int mode = mode_on(hb::kDrelu, dealer);
    if (mode < 0) return HB_EINVAL;
    return run(mode, share0, share1, n, k, m, seed, out0, out1, opened_bits, stream);
}

int hb_relu_ex(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed, int dealer,
               int64_t *out0, int64_t *out1, uint64_t *opened_bits, void *stream)
{
    const int mode = mode_on(hb::kRelu, dealer);
    if (mode < 0) return HB_EINVAL;
    return run(mode, share0, share1, n, k, m, seed, out0, out1, opened_bits, stream);
}

int hb_relu_batch_ex(const hb_tensor *tensors, size_t count, int dealer, uint64_t *opened_bits, void *stream)
{
    const int mode = mode_on(hb::kRelu, dealer);
    if (mode < 0) return HB_EINVAL;
    return run_batch(mode, tensors, count, opened_bits, stream);
}

int hb_drelu_batch_ex(const hb_tensor *tensors, size_t count, int dealer, uint64_t *opened_bits, void *stream)
{
    const int mode = mode_on(hb::kDrelu, dealer);
    if (mode < 0) return HB_EINVAL;
    return run_batch(mode, tensors, count, opened_bits, stream);
}

struct hb_plan {
    std::vector<LaunchItem> items;
    uint64_t opened_bits = 0;
};

int hb_plan_create(const hb_tensor *tensors, size_t count, int relu, int dealer, hb_plan **plan)
{
    if (plan == nullptr) return HB_EINVAL;
    *plan = nullptr;
    const int mode = mode_on(relu ? hb::kRelu : hb::kDrelu, dealer);
    if (mode < 0) return HB_EINVAL;
    uint64_t bits = 0;
    int st = validate_set(mode, tensors, count, &bits);
    if (st != HB_OK) return st;
    hb_plan *p = new (std::nothrow) hb_plan;
    if (p == nullptr) return HB_EINVAL;
    st = plan_launches(mode, tensors, count, p->items);
    if (st != HB_OK) {
        delete p;
        return st;
    }
    p->opened_bits = bits;
    *plan = p;
    return HB_OK;
}

int hb_plan_run(const hb_plan *plan, uint64_t *opened_bits, void *stream)
{
    if (plan == nullptr) return HB_EINVAL;
    for (const LaunchItem &it : plan->items) {
        const hipError_t e = enqueue(it, (hipStream_t)stream);
        if (e != hipSuccess) return fail_hip(e, "kernel launch");
    }
    if (opened_bits) *opened_bits = plan->opened_bits;
    return HB_OK;
}

void hb_plan_destroy(hb_plan *plan) { delete plan; }

int hb_drelu_mp(const int64_t *const *shares, int parties, size_t n, int k, int m, uint64_t seed,
                int64_t *const *outs, uint64_t *opened_bits, void *stream)
{
    return run_mp(hb::kDrelu, shares, parties, n, k, m, seed, outs, opened_bits, stream);
}

int hb_relu_mp(const int64_t *const *shares, int parties, size_t n, int k, int m, uint64_t seed,
               int64_t *const *outs, uint64_t *opened_bits, void *stream)
{
    return run_mp(hb::kRelu, shares, parties, n, k, m, seed, outs, opened_bits, stream);
}

size_t hb_party_wire_words(size_t n, int k, int m)
{
    if (!valid_slice(k, m) || n > HB_MAX_ELEMENTS) return 0;
    const PartyLayout lay = party_layout(n, k, m);
    return (size_t)lay.wire_words;
}

size_t hb_party_workspace_bytes(size_t n, int k, int m)
{
    if (!valid_slice(k, m) || n > HB_MAX_ELEMENTS) return 0;
    return (size_t)party_layout(n, k, m).total_bytes;
}

size_t hb_party_wire_offset(size_t n, int k, int m, int party)
{
    if (!valid_slice(k, m) || n > HB_MAX_ELEMENTS || party < 0 || party > 1) return 0;
    return (size_t)party_layout(n, k, m).wire_off[party];
}

int hb_relu_party(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed, int64_t *out0,
                  int64_t *out1, void *workspace, size_t workspace_bytes, uint64_t *wire_bytes, void *stream)
{
    return run_party(share0, share1, n, k, m, seed, HB_DEALER_PER_GATE, out0, out1, workspace, workspace_bytes, false,
                     wire_bytes, stream);
}

int hb_relu_party_ex(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed, int dealer,
                     int64_t *out0, int64_t *out1, void *workspace, size_t workspace_bytes, uint64_t *wire_bytes,
                     void *stream)
{
    return run_party(share0, share1, n, k, m, seed, dealer, out0, out1, workspace, workspace_bytes, false, wire_bytes,
                     stream);
}

size_t hb_party_wire_words_ex(size_t n, int k, int m, int dealer)
{
    if (!valid_slice(k, m) || n > HB_MAX_ELEMENTS || (dealer != HB_DEALER_PER_GATE && dealer != HB_DEALER_SHARED_MASK)) return 0;
    return (size_t)party_layout(n, k, m, dealer).wire_words;
}

size_t hb_party_workspace_bytes_ex(size_t n, int k, int m, int dealer)
{
    if (!valid_slice(k, m) || n > HB_MAX_ELEMENTS || (dealer != HB_DEALER_PER_GATE && dealer != HB_DEALER_SHARED_MASK)) return 0;
    return (size_t)party_layout(n, k, m, dealer).total_bytes;
}

size_t hb_party_wire_offset_ex(size_t n, int k, int m, int dealer, int party)
{
    if (!valid_slice(k, m) || n > HB_MAX_ELEMENTS || party < 0 || party > 1 ||
        (dealer != HB_DEALER_PER_GATE && dealer != HB_DEALER_SHARED_MASK))
        return 0;
    return (size_t)party_layout(n, k, m, dealer).wire_off[party];
}

int hb_relu_party_static(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed,
                         int64_t *out0, int64_t *out1, uint64_t *wire_bytes, void *stream)
{
    if (!valid_slice(k, m) || n > HB_MAX_ELEMENTS) return HB_EINVAL;
    if (party_layout(n, k, m).total_bytes > HB_PARTY_STATIC_BYTES) return HB_ETOOBIG;
    void *ws = nullptr;
    const int st = party_scratch_of_current_device(&ws);
    if (st != HB_OK) return st;
    return run_party(share0, share1, n, k, m, seed, HB_DEALER_PER_GATE, out0, out1, ws, HB_PARTY_STATIC_BYTES, true,
                     wire_bytes, stream);
}

int hb_share_f32(const float *x, size_t n, uint64_t share_seed, int64_t *share0, int64_t *share1, void *stream)
{
    const void *ptrs[2] = {share0, share1};
    int st = check_common(ptrs, 2, n);
    if (st != HB_OK) return st;
    if (n == 0) return HB_OK;
    st = check_float_buffer(x, n, 4);
    if (st != HB_OK) return st;
    const Range rx{(uintptr_t)x, (uintptr_t)x + 4 * n}, r0 = range_of(share0, n), r1 = range_of(share1, n);
    if (!disjoint(r0, r1) || !disjoint(rx, r0) || !disjoint(rx, r1)) return HB_EINVAL;
    const uint64_t blocks = ((uint64_t)n + hb::kBlock - 1) / hb::kBlock;
    if (blocks > 0x7fffffffull) return HB_EINVAL;
    hipLaunchKernelGGL(hb::share_f32_kernel, dim3((unsigned)blocks), dim3(hb::kBlock), 0, (hipStream_t)stream, x,
                       (uint64_t)n, share_seed, (uint64_t *)share0, (uint64_t *)share1);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? HB_OK : fail_hip(e, "kernel launch");
}

int hb_reveal_f32(const int64_t *share0, const int64_t *share1, size_t n, float *y, void *stream)
{
    const void *ptrs[2] = {share0, share1};
    int st = check_common(ptrs, 2, n);
    if (st != HB_OK) return st;
    if (n == 0) return HB_OK;
    st = check_float_buffer(y, n, 4);
    if (st != HB_OK) return st;
    const Range ry{(uintptr_t)y, (uintptr_t)y + 4 * n};
    if (!disjoint(ry, range_of(share0, n)) || !disjoint(ry, range_of(share1, n))) return HB_EINVAL;
    const uint64_t blocks = ((uint64_t)n + hb::kBlock - 1) / hb::kBlock;
    if (blocks > 0x7fffffffull) return HB_EINVAL;
    hipLaunchKernelGGL(hb::reveal_f32_kernel, dim3((unsigned)blocks), dim3(hb::kBlock), 0, (hipStream_t)stream,
                       (const uint64_t *)share0, (const uint64_t *)share1, (uint64_t)n, y);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? HB_OK : fail_hip(e, "kernel launch");
}

int hb_sim_relu_f32(const float *x, size_t n, int k, int m, uint64_t seed, uint64_t share_seed, float *y, void *stream)
{
    if (!valid_slice(k, m)) return HB_EINVAL;
    if (n > HB_MAX_ELEMENTS) return HB_EINVAL;
    const hb::SimLauncher f = hb::launcher_table().sim[m - k - 1];
    if (f == nullptr) return HB_ENOTSUP;
    if (n == 0) return HB_OK;
    int st = check_float_buffer(x, n, 8);
    if (st != HB_OK) return st;
    st = check_float_buffer(y, n, 8);
    if (st != HB_OK) return st;
    const Range rx{(uintptr_t)x, (uintptr_t)x + 4 * n}, ry{(uintptr_t)y, (uintptr_t)y + 4 * n};
    if (!(rx.lo == ry.lo || disjoint(rx, ry))) return HB_EINVAL;
    const hipError_t e = f(x, (uint64_t)n, k, hb::stream_word(seed, 0), hb::stream_word(seed, 1), share_seed, y,
                           (hipStream_t)stream);
    return e == hipSuccess ? HB_OK : fail_hip(e, "kernel launch");
}

int hb_eco_scan(const int64_t *share0, const int64_t *share1, size_t n, uint64_t *counts, void *stream)
{
    if (counts == nullptr) return HB_EINVAL;
    if (((uintptr_t)counts & 7u) != 0) return HB_EALIGN;
    const void *ptrs[2] = {share0, share1};
    int st = check_common(ptrs, 2, n);
    if (st != HB_OK) return st;
    st = check_device_buffer(counts, 64);
    if (st != HB_OK) return st;
    if (n > 0) {
        const Range c = range_of(counts, 64);
        if (!disjoint(c, range_of(share0, n)) || !disjoint(c, range_of(share1, n))) return HB_EINVAL;
    }
    hipLaunchKernelGGL(hb::eco_zero_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (unsigned long long *)counts);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    if (n == 0) return HB_OK;
    // aim at about 1024 wavefronts (one block per CU: the per-wave epilogue and the 64 atomics per block are
    // fixed costs, and 4 waves per CU with 64 loads in flight each already stream at 4.4 TB/s);
    // a lane takes `chunks` carry-save trees of 64 elements
    const uint64_t target_waves = 1024;
    uint64_t per_lane = ((uint64_t)n + target_waves * 64 - 1) / (target_waves * 64);
    uint64_t chunks = (per_lane + hb::kEcoChunk - 1) / hb::kEcoChunk;
    if (chunks < 1) chunks = 1;
    if (chunks > (uint64_t)hb::kEcoMaxPerLane / hb::kEcoChunk) chunks = hb::kEcoMaxPerLane / hb::kEcoChunk;
    const uint64_t per_wave = (uint64_t)hb::kWave * hb::kEcoChunk * chunks;
    const uint64_t waves = ((uint64_t)n + per_wave - 1) / per_wave;
    const uint64_t blocks = (waves + hb::kWavesPerBlock - 1) / hb::kWavesPerBlock;
    if (blocks > 0x7fffffffull) return HB_EINVAL;
    int live = 1;
    while ((1ull << live) <= chunks * hb::kEcoChunk) ++live;      // planes that can be non-zero
    if (all_aligned16(ptrs, 2)) {
        hipLaunchKernelGGL((hb::eco_scan_kernel<true>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, (hipStream_t)stream,
                           (const uint64_t *)share0, (const uint64_t *)share1, (uint64_t)n, (int)chunks, live,
                           (unsigned long long *)counts);
    } else {
        hipLaunchKernelGGL((hb::eco_scan_kernel<false>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, (hipStream_t)stream,
                           (const uint64_t *)share0, (const uint64_t *)share1, (uint64_t)n, (int)chunks, live,
                           (unsigned long long *)counts);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    return HB_OK;
}

int hb_eco_choose(const uint64_t *counts)
{
    if (counts == nullptr) return HB_EINVAL;
    int m = 64;
    while (m > 1 && counts[m - 2] == 0) --m;
    return m;
}

int hb_open(const int64_t *share0, const int64_t *share1, size_t n, int binary, int64_t *out, void *stream)
{
    const void *ptrs[3] = {share0, share1, out};
    const int st = check_common(ptrs, 3, n);
    if (st != HB_OK) return st;
    if (n == 0) return HB_OK;
    const Range i0 = range_of(share0, n), i1 = range_of(share1, n), r = range_of(out, n);
    if (!(same(r, i0) || disjoint(r, i0)) || !(same(r, i1) || disjoint(r, i1))) return HB_EINVAL;
    const bool vec = all_aligned16(ptrs, 3);
    const uint64_t threads = vec ? ((uint64_t)n + 1) / 2 : (uint64_t)n;
    const uint64_t blocks = (threads + hb::kBlock - 1) / hb::kBlock;
    if (blocks > 0x7fffffffull) return HB_EINVAL;
    if (vec) {
        hipLaunchKernelGGL((hb::open_kernel<true>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, (hipStream_t)stream,
                           (const uint64_t *)share0, (const uint64_t *)share1, (uint64_t)n, binary, (uint64_t *)out);
    } else {
        hipLaunchKernelGGL((hb::open_kernel<false>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, (hipStream_t)stream,
                           (const uint64_t *)share0, (const uint64_t *)share1, (uint64_t)n, binary, (uint64_t *)out);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    return HB_OK;
}

uint64_t hb_tensor_seed(uint64_t root_seed, uint64_t tensor_id) { return hb::stream_word(root_seed, 2 + tensor_id); }

uint64_t hb_opened_bits(int relu, int k, int m, size_t n)
{
    return hb_opened_bits_ex(relu, k, m, n, HB_DEALER_PER_GATE);
}

uint64_t hb_opened_bits_ex(int relu, int k, int m, size_t n, int dealer)
{
    if (!valid_slice(k, m) || (dealer != HB_DEALER_PER_GATE && dealer != HB_DEALER_SHARED_MASK)) return 0;
    const uint64_t w = (uint64_t)(m - k), R = (uint64_t)rounds_of((int)w);
    // gate 0 opens 2w bits; a prefix round opens 4w, or 3w when its two gates share the mask of P
    const uint64_t per_round = dealer == HB_DEALER_SHARED_MASK ? 3 * w : 4 * w;
    const uint64_t per = 2 * w + per_round * R + 1 + (relu ? 128 : 0);
    return (uint64_t)n * per;
}

uint64_t hb_opened_bits_mp(int relu, int parties, int k, int m, size_t n)
{
    if (!valid_slice(k, m) || parties < 2 || parties > hb::kMaxParties) return 0;
    const uint64_t w = (uint64_t)(m - k), R = (uint64_t)rounds_of((int)w);
    // per link and direction: parties - 1 adders of 1 + 2R gates, each opening 2w bits
    return (uint64_t)n * ((uint64_t)(parties - 1) * 2 * w * (1 + 2 * R) + 1 + (relu ? 128 : 0));
}

const char *hb_strerror(int status)
{
    switch (status) {
    case HB_OK: return "success";
    case HB_EINVAL: return "invalid argument (null pointer, bad (k, m), size, overlap, or not device memory)";
    case HB_EALIGN: return "pointer is not 8-byte aligned";
    case HB_EHIP: return "HIP runtime error (see hb_last_hip_error)";
    case HB_ENOTSUP: return "no kernel for this slice width in this entry point";
    case HB_ETOOBIG: return "the call needs more workspace than the library's static array holds";
    default: return "unknown status";
    }
}

const char *hb_last_hip_error(void) { return g_hip_error; }

}  // extern "C"
