// C ABI of the optgqa library: argument checks, launch-shape decisions, kernel dispatch.
// Declarations and the meaning of every argument: include/optgqa.h.
#include "optgqa.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <tuple>
#include <type_traits>
#include <utility>

#include "cache_kernels.hpp"
#include "decode_kernels.hpp"
#include "decode_mc_kernels.hpp"
#include "decode_mma_kernels.hpp"
#include "decode_flat_kernels.hpp"
#include "prefill_kernels.hpp"
#include "probe_kernels.hpp"

using namespace optgqa;

// Split-context scratch for optgqa_paged_attention_static, whose callers cannot allocate or
// bring a workspace.  One copy per GPU the library runs on, held until the process ends.  In
// host code this name is only a stand-in for the symbol: its device address comes from
// hipGetSymbolAddress (static_scratch() below) and is what kernels and size checks use.
static __device__ __align__(256) unsigned char g_static_scratch[OPTGQA_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kAbiVersion = 2;
constexpr int kMinPartition = 256;        // tokens; smaller runs are dominated by the merge

bool dtype_ok(int dt) { return dt == OPTGQA_F16 || dt == OPTGQA_BF16; }
bool head_dim_ok(int d) { return d == 64 || d == 128; }
bool block_size_ok(int bs) { return bs == 16 || bs == 32 || bs == 64; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Launch through the call that reports THIS launch's own status (hipLaunchKernel): an error
// some earlier work of the caller left behind in the runtime's "last error" slot is neither
// reported as ours nor cleared.
template <typename... KArgs, typename... Args>
int launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st, Args&&... args)
{
    static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count does not match the kernel");
    std::tuple<std::decay_t<KArgs>...> vals(std::forward<Args>(args)...);
    void* ptrs[sizeof...(KArgs)];
    std::apply([&](auto&... v) { int i = 0; ((ptrs[i++] = static_cast<void*>(&v)), ...); }, vals);
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, st) == hipSuccess
               ? OPTGQA_OK : OPTGQA_ERR_LAUNCH;
}

// Compute units of the current device, asked once (every GPU of a box is the same part); 256,
// the MI355X count, where no device answers (the sizing calls also work on a GPU-less host).
int num_cus()
{
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            return 256;
        return n;
    }();
    return cus;
}

// Profiling aid (optgqa_set_kernel_events): events recorded around the launch of the kernel that
// streams the KV cache, per calling thread.
thread_local hipEvent_t g_event_start = nullptr;
thread_local hipEvent_t g_event_stop = nullptr;

struct KernelEvents {
    hipStream_t st;
    explicit KernelEvents(hipStream_t s) : st(s)
    {
        if (g_event_start) (void)hipEventRecord(g_event_start, st);
    }
    ~KernelEvents()
    {
        if (g_event_stop) (void)hipEventRecord(g_event_stop, st);
    }
};

// Device address of g_static_scratch on the current device, looked up once per device (each GPU
// holds its own copy at its own address).  nullptr if the runtime refuses.
constexpr int kMaxDevices = 64;
void* static_scratch()
{
    static std::mutex mu;
    static void* ptr[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess) return nullptr;
        ptr[dev] = p;
    }
    return ptr[dev];
}

// Number of query heads one workgroup serves from a single pass over its K/V tiles; always a
// divisor of the group size.  The matrix-core kernels (head_dim 128 unsplit, and the equal-work
// kernel at either head_dim) have a score tile of 16 columns: the largest divisor <= 16.  The
// head_dim 64 kernels that run unsplit: the largest of 8, 4, 2, 1.
int mfma_heads_per_workgroup(int group)
{
    for (int gh = group < kMmaMaxHeads ? group : kMmaMaxHeads; gh > 1; --gh)
        if (group % gh == 0) return gh;
    return 1;
}

int heads_per_workgroup(int group, int head_dim)
{
    if (head_dim == 128) return mfma_heads_per_workgroup(group);
    for (int gh = 8; gh > 1; gh >>= 1)
        if (group % gh == 0) return gh;
    return 1;
}

int round_up(int x, int m) { return (x + m - 1) / m * m; }

// Partition size the library picks when the caller leaves the choice to it (0 = do not split).
// Aim: enough workgroups to occupy every CU several times over, runs no shorter than
// kMinPartition tokens.
int auto_partition(int num_seqs, int num_heads, int num_kv_heads, int head_dim, int block_size,
                   int max_context_len)
{
    if (max_context_len <= kMinPartition) return 0;
    const int group = num_heads / num_kv_heads;
    const long units = (long)num_seqs * num_kv_heads * (group / heads_per_workgroup(group, head_dim));
    const long want_wgs = 8L * num_cus();
    if (units >= want_wgs) return 0;
    long np = (want_wgs + units - 1) / units;                       // partitions per sequence
    int step = block_size > 16 ? block_size : 16;
    if (kMinPartition % step) step = kMinPartition;                  // keep P a multiple of both
    int P = round_up((int)((max_context_len + np - 1) / np), step);
    if (P < kMinPartition) P = kMinPartition;
    if (P >= max_context_len) return 0;
    return P;
}

// Rows are sequences.  A launch covers at most kMaxRowsPerLaunch rows because grid.y / grid.z
// are 16-bit.
constexpr int kMaxRowsPerLaunch = 65535;

struct SplitPlan {
    int partition_size;   // 0 = unsplit, OPTGQA_SPLIT_BALANCED = equal-work split
    int num_partitions;
    size_t bytes;
    // equal-work kernel only (the equal-work split, and fixed partitions that are multiples of 16 tokens)
    int workgroups;
    int segs_per_seq;
    size_t plan_floats, ml_floats;
    int64_t slots;        // partial-result slots
    bool flat;            // the equal-work kernel runs this plan
};

// Equal-work split: one workgroup per CU for 2-byte caches (one wave per SIMD streams best),
// OPTGQA_FLAT_WGS_PER_CU_KV8 per CU for 8-bit caches (half the bytes per tile: the second wave
// per SIMD hides the arithmetic); no wave with less than kFlatMinTiles tiles of 16 tokens when
// the lengths are at their bound.  The workspace is sized for the larger of the two.
int flat_workgroups(bool kv8) { return num_cus() * (kv8 ? OPTGQA_FLAT_WGS_PER_CU_KV8 : OPTGQA_FLAT_WGS_PER_CU); }
int flat_max_workgroups() { return std::max(flat_workgroups(false), flat_workgroups(true)); }
#ifndef OPTGQA_FLAT_MIN_TILES
#define OPTGQA_FLAT_MIN_TILES 8
#endif
constexpr int kFlatMinTiles = OPTGQA_FLAT_MIN_TILES;

size_t round_up4(size_t x) { return (x + 3) / 4 * 4; }

// (shared: the flat order runs over two virtual sequences per sequence - a bundle's shared prefix
// and a sequence's own part - and every slot holds 16 columns, see decode_flat_kernels.hpp)
bool plan_flat(SplitPlan& s, int num_seqs, int num_heads, int num_kv_heads, int head_dim, int max_context_len,
               int window = 0, bool shared = false)
{
    const int group = num_heads / num_kv_heads;
    const int gh = mfma_heads_per_workgroup(group);
    const int64_t Y = (int64_t)num_kv_heads * (group / gh);
    const int64_t segs = Y * num_seqs * (shared ? 2 : 1);
    const int cols = shared ? 16 : gh;
    // Flat tile indices are 32-bit.  2^30 tiles would be 8 TiB of cache, so the margin of 2 also
    // covers lengths above the stated bound.
    if (segs * ((max_context_len + kMmaTile - 1) / kMmaTile) >= (1LL << 30)) return false;
    // tiles that will be read: with a sliding window at most window + 15 tokens per segment
    const int seen = window > 0 && window + kMmaTile - 1 < max_context_len ? window + kMmaTile - 1 : max_context_len;
    const int64_t tiles = Y * num_seqs * ((seen + kMmaTile - 1) / kMmaTile);
    int64_t wgs = (tiles + (int64_t)kDecodeWaves * kFlatMinTiles - 1) / ((int64_t)kDecodeWaves * kFlatMinTiles);
    if (wgs > flat_max_workgroups()) wgs = flat_max_workgroups();
    if (wgs < 1) wgs = 1;
    s.partition_size = OPTGQA_SPLIT_BALANCED;
    s.num_partitions = 1;
    s.workgroups = (int)wgs;
    s.segs_per_seq = (int)Y;
    const size_t slots = (size_t)wgs * kDecodeWaves + (size_t)segs;
    s.plan_floats = round_up4((size_t)num_seqs * (shared ? 2 : 1) + 1);
    s.ml_floats = round_up4(slots * cols);
    s.bytes = (s.plan_floats + 2 * s.ml_floats + slots * cols * head_dim) * sizeof(float);
    s.slots = (int64_t)slots;
    s.flat = true;
    return true;
}

// Fixed partitions of P tokens (a multiple of 16) run by the equal-work kernel: two partial-result
// slots per partition of every (sequence, KV head / head chunk) segment (a unit boundary may cut a
// partition in two).
bool plan_flat_parts(SplitPlan& s, int num_seqs, int num_heads, int num_kv_heads, int head_dim, int max_context_len, int P)
{
    const int group = num_heads / num_kv_heads;
    const int gh = mfma_heads_per_workgroup(group);
    const int64_t Y = (int64_t)num_kv_heads * (group / gh);
    const int np = (max_context_len + P - 1) / P;
    const int64_t parts = Y * num_seqs * np;                 // upper bound: every sequence at max_context_len
    if (parts * (P / kMmaTile) >= (1LL << 30)) return false;  // flat tile indices are 32-bit
    int64_t wgs = (parts + kDecodeWaves - 1) / kDecodeWaves;  // no more units than partitions
    if (wgs > flat_workgroups(false)) wgs = flat_workgroups(false);
    s.partition_size = P;
    s.num_partitions = np;
    s.workgroups = (int)wgs;
    s.segs_per_seq = (int)Y;
    s.slots = 2 * parts;
    s.plan_floats = round_up4((size_t)num_seqs + 1);
    s.ml_floats = round_up4((size_t)s.slots * gh);
    s.bytes = (s.plan_floats + 2 * s.ml_floats + (size_t)s.slots * gh * head_dim) * sizeof(float);
    s.flat = true;
    return true;
}

SplitPlan plan_split(int num_seqs, int num_heads, int num_kv_heads, int head_dim, int block_size,
                     int max_context_len, int partition_size, int window = 0, bool shared = false)
{
    SplitPlan s{0, 1, 0, 0, 0, 0, 0, 0, false};
    int P = partition_size;
    if (P == 0) P = auto_partition(num_seqs, num_heads, num_kv_heads, head_dim, block_size, max_context_len);
    // The library's own choice is the equal-work split whenever splitting pays.
    if (partition_size == OPTGQA_SPLIT_BALANCED || (partition_size == 0 && P > 0)) {
        if (plan_flat(s, num_seqs, num_heads, num_kv_heads, head_dim, max_context_len, window, shared))
            return s;
        if (partition_size == OPTGQA_SPLIT_BALANCED) return s;      // cannot: the caller sees "unsplit"
    }
    // fixed partitions (multiples of 16 tokens: checked by the caller) run on the same kernel
    if (partition_size > 0 && window <= 0 && !shared)
        plan_flat_parts(s, num_seqs, num_heads, num_kv_heads, head_dim, max_context_len, P);
    return s;                                                // (unsplit if that could not be planned)
}

// The fast decode kernel takes its LDS as dynamic shared memory (the ring may exceed the 64 KiB
// a kernel gets by default); the size limit is raised once per kernel instantiation.
template <int DT, int D, int GH>
int launch_decode_mc(const DecodeParams& p, dim3 grid, dim3 block, hipStream_t st)
{
    constexpr int kBytes = McSmem<D, GH>::kBytes;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&paged_decode_mc_kernel<DT, D, GH>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kBytes);
    if (attr != hipSuccess) return OPTGQA_ERR_LAUNCH;
    return launch(paged_decode_mc_kernel<DT, D, GH>, grid, block, kBytes, st, p);
}

template <int DT, int D>
int launch_decode_gh(const DecodeParams& p, int gh, dim3 grid, hipStream_t st)
{
    const dim3 block(kDecodeWaves * 64);
    if (D == 128) {
        return launch(paged_decode_mma_kernel<DT>, grid, block, 0, st, p);
    }
#ifndef OPTGQA_VALU_ONLY_DECODE
    if (gh == 8) return launch_decode_mc<DT, D, 8>(p, grid, block, st);
    if (gh == 4) return launch_decode_mc<DT, D, 4>(p, grid, block, st);
#endif
    switch (gh) {
    case 8: return launch(paged_decode_kernel<DT, D, 8>, grid, block, 0, st, p);
    case 4: return launch(paged_decode_kernel<DT, D, 4>, grid, block, 0, st, p);
    case 2: return launch(paged_decode_kernel<DT, D, 2>, grid, block, 0, st, p);
    default: return launch(paged_decode_kernel<DT, D, 1>, grid, block, 0, st, p);
    }
}


template <int DT, int D>
int launch_decode(DecodeParams p, int num_rows, hipStream_t st)
{
    const int group = p.num_heads / p.num_kv_heads;
    const int gh = heads_per_workgroup(group, D);
    p.heads_per_wg = gh;
    for (int first = 0; first < num_rows; first += kMaxRowsPerLaunch) {
        const int rows = num_rows - first < kMaxRowsPerLaunch ? num_rows - first : kMaxRowsPerLaunch;
        p.row_offset = first;
        const dim3 grid(1, p.num_kv_heads * (group / gh), rows);
        int rc;
        {
            KernelEvents ev(st);
            rc = launch_decode_gh<DT, D>(p, gh, grid, st);
        }
        if (rc != OPTGQA_OK) return rc;
    }
    return OPTGQA_OK;
}

template <typename... A>
int launch_decode_any(int dtype, int head_dim, A... args)
{
    if (dtype == OPTGQA_F16)
        return head_dim == 128 ? launch_decode<kF16, 128>(args...) : launch_decode<kF16, 64>(args...);
    return head_dim == 128 ? launch_decode<kBF16, 128>(args...) : launch_decode<kBF16, 64>(args...);
}

// Equal-work kernel: `workgroups` was sized for the work; it is also capped by what
// the device keeps resident at once, because a unit that has to wait for a free slot would start
// when every other unit is nearly done.
template <int DT, int D, bool FUSED, bool KV8 = false, bool SHARED = false, bool PARTS = false>
int launch_decode_flat_dt(DecodeParams p, int workgroups, hipStream_t st)
{
    static const int resident = [] {
        int per_cu = 0, dev = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, paged_decode_flat_kernel<DT, FUSED, KV8, SHARED, PARTS, D>, kDecodeWaves * 64, 0) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return 0;
        return per_cu * cus;
    }();
    if (resident <= 0) return OPTGQA_ERR_LAUNCH;
    if (workgroups > resident) workgroups = resident;
    const int group = p.num_heads / p.num_kv_heads;
    p.heads_per_wg = mfma_heads_per_workgroup(group);
    p.num_units = workgroups * kDecodeWaves;
    int rc;
    {
        KernelEvents ev(st);
        rc = launch(paged_decode_flat_kernel<DT, FUSED, KV8, SHARED, PARTS, D>, dim3(workgroups), dim3(kDecodeWaves * 64), 0, st, p);
    }
    if (rc != OPTGQA_OK) return rc;
    if constexpr (PARTS)
        return launch(paged_decode_parts_reduce_kernel<DT, D>, dim3(p.num_seqs, p.num_heads), dim3(kPartsReduceGroups * (D / 4)), 0, st, p);
    constexpr int kHeadsPerWg = kReduceThreads / (D / 4);
    return launch(paged_decode_flat_reduce_kernel<DT, FUSED && KV8, SHARED, D>, dim3(p.num_seqs, (p.num_heads + kHeadsPerWg - 1) / kHeadsPerWg),
                  dim3(kReduceThreads), 0, st, p);
}

template <int DT, int D>
int launch_decode_flat_d(const DecodeParams& p, int workgroups, hipStream_t st, bool kv8)
{
    if (p.part_tiles > 0) return launch_decode_flat_dt<DT, D, false, false, false, true>(p, workgroups, st);
    if (p.shared_blocks && p.k_new) return launch_decode_flat_dt<DT, D, true, false, true>(p, workgroups, st);
    if (p.shared_blocks) return launch_decode_flat_dt<DT, D, false, false, true>(p, workgroups, st);
    if (kv8 && p.k_new) return launch_decode_flat_dt<DT, D, true, true>(p, workgroups, st);
    if (kv8) return launch_decode_flat_dt<DT, D, false, true>(p, workgroups, st);
    if (p.k_new) return launch_decode_flat_dt<DT, D, true>(p, workgroups, st);
    return launch_decode_flat_dt<DT, D, false>(p, workgroups, st);
}

int launch_decode_flat(int dtype, int head_dim, const DecodeParams& p, int workgroups, hipStream_t st, bool kv8 = false)
{
    if (head_dim == 128)
        return dtype == OPTGQA_F16 ? launch_decode_flat_d<kF16, 128>(p, workgroups, st, kv8)
                                   : launch_decode_flat_d<kBF16, 128>(p, workgroups, st, kv8);
    return dtype == OPTGQA_F16 ? launch_decode_flat_d<kF16, 64>(p, workgroups, st, kv8)
                               : launch_decode_flat_d<kBF16, 64>(p, workgroups, st, kv8);
}


// The tiled prefill kernel takes its LDS as dynamic shared memory (more than the 64 KiB a kernel
// gets by default); the limit is raised once per instantiation.
template <int DT, bool KV8, bool WIN, bool CONTIG, int D, int WAVES>
int launch_prefill_mma_w(const PrefillParams& p, dim3 grid, hipStream_t st)
{
    constexpr int kBytes = PfTile<D>::kLdsBytes;
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(&paged_prefill_mma_kernel<DT, KV8, WIN, CONTIG, D, WAVES>),
        hipFuncAttributeMaxDynamicSharedMemorySize, kBytes);
    if (attr != hipSuccess) return OPTGQA_ERR_LAUNCH;
    return launch(paged_prefill_mma_kernel<DT, KV8, WIN, CONTIG, D, WAVES>, grid, dim3(WAVES * 64), kBytes, st, p);
}

template <int DT, bool KV8, bool WIN, bool CONTIG, int D>
int launch_prefill_mma_d(const PrefillParams& p, dim3 grid, int waves, hipStream_t st)
{
    if constexpr (!WIN) {
        if (waves == 8) return launch_prefill_mma_w<DT, KV8, WIN, CONTIG, D, 8>(p, grid, st);
    }
    return launch_prefill_mma_w<DT, KV8, WIN, CONTIG, D, 4>(p, grid, st);
}

template <int DT, bool KV8, bool WIN, bool CONTIG>
int launch_prefill_mma(const PrefillParams& p, int head_dim, dim3 grid, int waves, hipStream_t st)
{
    if (head_dim == 64) return launch_prefill_mma_d<DT, KV8, WIN, CONTIG, 64>(p, grid, waves, st);
    return launch_prefill_mma_d<DT, KV8, WIN, CONTIG, 128>(p, grid, waves, st);
}

// The one-call prefill step (cache write inside the prefill kernel).
template <int DT, int D, int WAVES>
int launch_prefill_step_w(const PrefillParams& p, dim3 grid, hipStream_t st)
{
    constexpr int kBytes = PfTile<D>::kLdsBytes;
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(&paged_prefill_step_kernel<DT, D, WAVES>),
        hipFuncAttributeMaxDynamicSharedMemorySize, kBytes);
    if (attr != hipSuccess) return OPTGQA_ERR_LAUNCH;
    return launch(paged_prefill_step_kernel<DT, D, WAVES>, grid, dim3(WAVES * 64), kBytes, st, p);
}

template <int DT>
int launch_prefill_step(const PrefillParams& p, int head_dim, dim3 grid, int waves, hipStream_t st)
{
    if (head_dim == 64)
        return waves == 8 ? launch_prefill_step_w<DT, 64, 8>(p, grid, st) : launch_prefill_step_w<DT, 64, 4>(p, grid, st);
    return waves == 8 ? launch_prefill_step_w<DT, 128, 8>(p, grid, st) : launch_prefill_step_w<DT, 128, 4>(p, grid, st);
}

// The tiled prefill kernel carries the tile-invariant part of the ALiBi term inside the score
// accumulator as slope / scale, so it cannot take a score scale of exactly zero.  Magnitudes
// below 2^-64 (zero included) are evaluated as +-2^-64: the scores then differ from the exact
// ones by |q.k| * 2^-64, far below fp32 resolution of the bias they are added to.
float prefill_scale2(float scale)
{
    const float tiny = 0x1p-64f;
    const float s = std::fabs(scale) < tiny ? std::copysign(tiny, scale) : scale;
    return s * kLog2e;
}

// Tiled matrix-core prefill (head_dim 128 or 64).
int launch_prefill(PrefillParams p, int num_seqs, int max_q_len, int head_dim, int dtype, hipStream_t st,
                   bool kv8 = false, bool contig = false, bool step = false)
{
    if (head_dim != 128 && head_dim != 64) return OPTGQA_ERR_UNSUPPORTED;
    const int group = p.num_heads / p.num_kv_heads;
    const int gh = mfma_heads_per_workgroup(group);
    int shift = 0;
    while ((1 << shift) < gh) ++shift;
    p.num_seqs = num_seqs;
    p.heads_per_wg = gh;
    p.heads_pow2_shift = shift;
    p.units = num_seqs * p.num_kv_heads * (group / gh);
    // 8 waves per workgroup when that still leaves two rounds of workgroups per CU, else 4 (and 4
    // with a sliding window): see prefill_kernels.hpp
    const int64_t units8 = (p.units + 7) / 8 * 8;
    const int tokens_per_wg8 = (8 * 32) >> shift;
    const int64_t blocks8 = units8 * ((max_q_len + tokens_per_wg8 - 1) / tokens_per_wg8);
    const int waves = (p.window > 0 || blocks8 < 2 * num_cus()) ? 4 : 8;
    const int tokens_per_wg = (waves * 32) >> shift;
    p.q_tiles = (max_q_len + tokens_per_wg - 1) / tokens_per_wg;
    const int64_t blocks = units8 * p.q_tiles;
    if (blocks > 0x7fffffffLL) return OPTGQA_ERR_SHAPE;
    const dim3 grid((unsigned)blocks);
    KernelEvents ev(st);
    const bool f16 = dtype == OPTGQA_F16;
    if (step) {
        if (kv8 || contig || p.window > 0) return OPTGQA_ERR_UNSUPPORTED;
        return f16 ? launch_prefill_step<kF16>(p, head_dim, grid, waves, st)
                   : launch_prefill_step<kBF16>(p, head_dim, grid, waves, st);
    }
    if (contig) {
        if (kv8 || p.window > 0) return OPTGQA_ERR_UNSUPPORTED;
        return f16 ? launch_prefill_mma<kF16, false, false, true>(p, head_dim, grid, waves, st)
                   : launch_prefill_mma<kBF16, false, false, true>(p, head_dim, grid, waves, st);
    }
    if (p.window > 0) {
        if (kv8) return OPTGQA_ERR_UNSUPPORTED;
        return f16 ? launch_prefill_mma<kF16, false, true, false>(p, head_dim, grid, waves, st)
                   : launch_prefill_mma<kBF16, false, true, false>(p, head_dim, grid, waves, st);
    }
    if (kv8)
        return f16 ? launch_prefill_mma<kF16, true, false, false>(p, head_dim, grid, waves, st)
                   : launch_prefill_mma<kBF16, true, false, false>(p, head_dim, grid, waves, st);
    return f16 ? launch_prefill_mma<kF16, false, false, false>(p, head_dim, grid, waves, st)
               : launch_prefill_mma<kBF16, false, false, false>(p, head_dim, grid, waves, st);
}

}  // namespace


extern "C" {

int optgqa_abi_version(void) { return kAbiVersion; }

int optgqa_set_kernel_events(void* start_event, void* stop_event)
{
    if ((start_event == nullptr) != (stop_event == nullptr)) return OPTGQA_ERR_NULL;
    g_event_start = static_cast<hipEvent_t>(start_event);
    g_event_stop = static_cast<hipEvent_t>(stop_event);
    return OPTGQA_OK;
}

const char* optgqa_status_string(int status)
{
    switch (status) {
    case OPTGQA_OK: return "ok";
    case OPTGQA_ERR_NULL: return "a required pointer is NULL";
    case OPTGQA_ERR_SHAPE: return "inconsistent or non-positive sizes";
    case OPTGQA_ERR_UNSUPPORTED: return "unsupported head_dim, block_size, dtype or alignment";
    case OPTGQA_ERR_WORKSPACE: return "workspace missing or too small for the split-context path";
    case OPTGQA_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    case OPTGQA_ERR_TABLE: return "block table or context length out of range";
    default: return "unknown status";
    }
}

int optgqa_reshape_and_cache(const void* k, const void* v, void* k_cache, void* v_cache,
                             const int64_t* slot_mapping, int num_tokens, int num_kv_heads,
                             int head_dim, int block_size, int64_t k_token_stride,
                             int64_t v_token_stride, int dtype, void* stream)
{
    if (num_tokens < 0 || num_kv_heads <= 0 || head_dim <= 0 || block_size <= 0) return OPTGQA_ERR_SHAPE;
    if (!dtype_ok(dtype) || !head_dim_ok(head_dim) || !block_size_ok(block_size)) return OPTGQA_ERR_UNSUPPORTED;
    const int64_t row = (int64_t)num_kv_heads * head_dim;
    if (k_token_stride < row || v_token_stride < row) return OPTGQA_ERR_SHAPE;
    if (num_tokens == 0) return OPTGQA_OK;
    if (!k || !v || !k_cache || !v_cache || !slot_mapping) return OPTGQA_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(k) | reinterpret_cast<uintptr_t>(v) |
         reinterpret_cast<uintptr_t>(k_cache) | reinterpret_cast<uintptr_t>(v_cache)) & 1u)
        return OPTGQA_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool wide = aligned16(k) && aligned16(v) && aligned16(k_cache) && aligned16(v_cache) &&
                      k_token_stride % 8 == 0 && v_token_stride % 8 == 0;
    const int elems = wide ? 8 : 1;
    const int64_t threads = (int64_t)num_tokens * num_kv_heads * (head_dim / elems) * 2;
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffLL) return OPTGQA_ERR_SHAPE;
    auto kk = static_cast<const uint16_t*>(k);
    auto vv = static_cast<const uint16_t*>(v);
    auto kc = static_cast<uint16_t*>(k_cache);
    auto vc = static_cast<uint16_t*>(v_cache);
    return launch(wide ? reshape_and_cache_kernel<uint4> : reshape_and_cache_kernel<uint16_t>, dim3((unsigned)blocks),
                  dim3(256), 0, st, kk, vv, kc, vc, slot_mapping, num_tokens, num_kv_heads, head_dim, block_size,
                  k_token_stride, v_token_stride, nullptr, nullptr, 0);
}

size_t optgqa_paged_attention_workspace_bytes(int num_seqs, int num_heads, int num_kv_heads,
                                              int head_dim, int block_size, int max_context_len,
                                              int partition_size, int* chosen_partition_size)
{
    if (chosen_partition_size) *chosen_partition_size = 0;
    if (num_seqs <= 0 || num_heads <= 0 || num_kv_heads <= 0 || head_dim <= 0 || block_size <= 0 ||
        max_context_len <= 0 || num_heads % num_kv_heads)
        return 0;
    const SplitPlan s = plan_split(num_seqs, num_heads, num_kv_heads, head_dim, block_size,
                                   max_context_len, partition_size);
    if (chosen_partition_size) *chosen_partition_size = s.partition_size;
    return s.bytes;
}

}  // extern "C"

namespace {

// Scales of 8-bit (E4M3) caches: one pair per tensor (k, v), or - k_heads / v_heads set, device
// arrays of num_kv_heads values each - one pair per KV head.
struct KvScales {
    float k, v;
    const float* k_heads;
    const float* v_heads;
    bool per_head() const { return k_heads != nullptr; }
    bool valid() const
    {
        if (per_head()) return v_heads != nullptr;           // contents live on the device: not checked here
        return k > 0.f && v > 0.f && k <= 3e38f && v <= 3e38f;
    }
};

// New-token inputs of a fused decode step (all null / zero for plain attention).
struct StepInputs {
    const void* k_new;
    const void* v_new;
    int64_t k_stride, v_stride;
    void* k_cache_w;
    void* v_cache_w;
};

int write_new_tokens(const StepInputs& n, const int64_t* slot_mapping, const int32_t* block_tables,
                     const int32_t* context_lens, int num_tokens, int num_kv_heads, int head_dim, int block_size,
                     int max_blocks_per_seq, hipStream_t st)
{
    const bool wide = aligned16(n.k_new) && aligned16(n.v_new) && aligned16(n.k_cache_w) && aligned16(n.v_cache_w) &&
                      n.k_stride % 8 == 0 && n.v_stride % 8 == 0;
    const int elems = wide ? 8 : 1;
    const int64_t threads = (int64_t)num_tokens * num_kv_heads * (head_dim / elems) * 2;
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffLL) return OPTGQA_ERR_SHAPE;
    auto kk = static_cast<const uint16_t*>(n.k_new);
    auto vv = static_cast<const uint16_t*>(n.v_new);
    auto kc = static_cast<uint16_t*>(n.k_cache_w);
    auto vc = static_cast<uint16_t*>(n.v_cache_w);
    return launch(wide ? reshape_and_cache_kernel<uint4> : reshape_and_cache_kernel<uint16_t>, dim3((unsigned)blocks),
                  dim3(256), 0, st, kk, vv, kc, vc, slot_mapping, num_tokens, num_kv_heads, head_dim, block_size,
                  n.k_stride, n.v_stride, block_tables, context_lens, max_blocks_per_seq);
}

// Decode attention, optionally preceded by (or fused with) the step's cache write.
int attention_impl(void* out, const void* q, const void* k_cache, const void* v_cache,
                   const int32_t* block_tables, const int32_t* context_lens, const float* alibi_slopes,
                   float scale, int num_seqs, int num_heads, int num_kv_heads, int head_dim, int block_size,
                   int max_blocks_per_seq, int max_context_len, int partition_size, void* workspace,
                   size_t workspace_bytes, int dtype, hipStream_t st, const StepInputs* step,
                   const KvScales* kv_scales = nullptr,   // the caches hold E4M3 codes with these scales
                   int window = 0,                        // > 0: sliding window (Alg. 1, local mask)
                   const int32_t* shared_blocks = nullptr) // shared prefixes, read once per bundle of sequences
{
    if (shared_blocks) {
        if (kv_scales || window > 0) return OPTGQA_ERR_UNSUPPORTED;
        partition_size = OPTGQA_SPLIT_BALANCED;          // the equal-work kernel only
    }
    if (window > 0) partition_size = OPTGQA_SPLIT_BALANCED;
    if (kv_scales) {
        if (kv_scales->per_head() && !kv_scales->v_heads) return OPTGQA_ERR_NULL;
        if (!kv_scales->valid()) return OPTGQA_ERR_SHAPE;
        partition_size = OPTGQA_SPLIT_BALANCED;          // the only kernel that reads E4M3 caches
    }
    if (num_seqs < 0 || num_heads <= 0 || num_kv_heads <= 0 || head_dim <= 0 || block_size <= 0 ||
        max_blocks_per_seq <= 0 || max_context_len < 0)
        return OPTGQA_ERR_SHAPE;
    if (!std::isfinite(scale)) return OPTGQA_ERR_SHAPE;
    if (num_heads % num_kv_heads) return OPTGQA_ERR_SHAPE;
    if ((int64_t)max_context_len > (int64_t)max_blocks_per_seq * block_size) return OPTGQA_ERR_SHAPE;
    if (!dtype_ok(dtype) || !head_dim_ok(head_dim) || !block_size_ok(block_size)) return OPTGQA_ERR_UNSUPPORTED;
    if (partition_size > 0 && (partition_size % block_size || partition_size % 16)) return OPTGQA_ERR_SHAPE;
    if (step) {
        const int64_t row = (int64_t)num_kv_heads * head_dim;
        if (step->k_stride < row || step->v_stride < row) return OPTGQA_ERR_SHAPE;
    }
    if (num_seqs == 0) return OPTGQA_OK;
    if (!out || !q || !k_cache || !v_cache || !block_tables || !context_lens) return OPTGQA_ERR_NULL;
    if (step && (!step->k_new || !step->v_new)) return OPTGQA_ERR_NULL;
    if (!aligned16(out) || !aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache)) return OPTGQA_ERR_UNSUPPORTED;
    if (step && ((reinterpret_cast<uintptr_t>(step->k_new) | reinterpret_cast<uintptr_t>(step->v_new)) & 1u))
        return OPTGQA_ERR_UNSUPPORTED;
    if (num_heads > 65535) return OPTGQA_ERR_SHAPE;

    SplitPlan s = plan_split(num_seqs, num_heads, num_kv_heads, head_dim, block_size,
                             max_context_len > 0 ? max_context_len : 1, partition_size, window, shared_blocks != nullptr);
    if (partition_size == OPTGQA_SPLIT_BALANCED && s.partition_size != OPTGQA_SPLIT_BALANCED)
        return OPTGQA_ERR_UNSUPPORTED;                   // sizes beyond 32-bit tile indices
    if (s.partition_size != 0) {
        const bool have = workspace && workspace_bytes >= s.bytes && aligned16(workspace);
        if (!have) {
            if (partition_size != 0) return OPTGQA_ERR_WORKSPACE;
            s = SplitPlan{0, 1, 0, 0, 0, 0, 0, 0, false};          // library's own choice: fall back to unsplit
        }
    }

    DecodeParams p;
    p.out = out;
    p.q = q;
    p.k_cache = k_cache;
    p.v_cache = v_cache;
    p.block_tables = block_tables;
    p.context_lens = context_lens;
    p.slopes = alibi_slopes;
    p.scale2 = scale * kLog2e;
    p.num_heads = num_heads;
    p.num_kv_heads = num_kv_heads;
    p.block_size = block_size;
    p.max_blocks_per_seq = max_blocks_per_seq;
    p.num_seqs = num_seqs;
    p.row_offset = 0;
    p.k_new = p.v_new = nullptr;
    p.k_cache_w = p.v_cache_w = nullptr;
    p.k_new_stride = p.v_new_stride = 0;
    p.out_scale = 1.f;
    p.window = window > 0 ? window : 0;
    p.new_token_in_combine = 0;
    p.k_inv_scale = p.v_inv_scale = 1.f;
    p.part_tiles = 0;
    p.shared_blocks = shared_blocks;
    p.bundle = shared_blocks ? kMmaMaxHeads / mfma_heads_per_workgroup(num_heads / num_kv_heads) : 1;
    p.k_scales = p.v_scales = nullptr;
    if (kv_scales && kv_scales->per_head()) {
        p.k_scales = kv_scales->k_heads;                     // applied per KV head inside the kernels
        p.v_scales = kv_scales->v_heads;
        p.new_token_in_combine = step != nullptr;
    } else if (kv_scales) {
        p.scale2 *= kv_scales->k;
        p.out_scale = kv_scales->v;
        p.k_inv_scale = 1.0f / kv_scales->k;                 // one fp32 division each, as the cache write does
        p.v_inv_scale = 1.0f / kv_scales->v;
        p.new_token_in_combine = step != nullptr;
    }

    // The cache write rides inside the equal-work kernel when that kernel runs and the new rows
    // can be moved as 16-byte pieces; otherwise it is a launch of its own ahead of the attention.
    bool fused = false;
    if (step) {
        fused = s.flat && s.partition_size == OPTGQA_SPLIT_BALANCED && aligned16(step->k_new) && aligned16(step->v_new) &&
                step->k_stride % 8 == 0 && step->v_stride % 8 == 0;
        if (!fused && kv_scales) return OPTGQA_ERR_UNSUPPORTED;   // 8-bit step: new rows must move as 16-byte pieces
        if (!fused) {
            const int rc = write_new_tokens(*step, nullptr, block_tables, context_lens, num_seqs, num_kv_heads,
                                            head_dim, block_size, max_blocks_per_seq, st);
            if (rc != OPTGQA_OK) return rc;
        }
    }

    if (s.flat) {
        p.plan = static_cast<int32_t*>(workspace);
        p.ws_m = static_cast<float*>(workspace) + s.plan_floats;
        p.ws_l = p.ws_m + s.ml_floats;
        p.ws_o = p.ws_l + s.ml_floats;
        p.num_partitions = 1;
        if (s.partition_size > 0) {                          // fixed partitions
            p.part_tiles = s.partition_size / kMmaTile;
            p.num_partitions = s.num_partitions;
        }
        p.segs_per_seq = s.segs_per_seq;
        if (fused) {
            p.k_new = step->k_new;
            p.v_new = step->v_new;
            p.k_new_stride = step->k_stride;
            p.v_new_stride = step->v_stride;
            p.k_cache_w = step->k_cache_w;
            p.v_cache_w = step->v_cache_w;
        }
        const int cap = flat_workgroups(kv_scales != nullptr);
        return launch_decode_flat(dtype, head_dim, p, s.workgroups < cap ? s.workgroups : cap, st, kv_scales != nullptr);
    }
    // unsplit: one workgroup per (sequence, KV head / head chunk) walks the whole context
    p.plan = nullptr;
    p.num_units = p.segs_per_seq = 0;
    p.ws_m = p.ws_l = p.ws_o = nullptr;
    p.num_partitions = 1;
    return launch_decode_any(dtype, head_dim, p, num_seqs, st);
}

}  // namespace

extern "C" {

int optgqa_paged_attention(void* out, const void* q, const void* k_cache, const void* v_cache,
                           const int32_t* block_tables, const int32_t* context_lens,
                           const float* alibi_slopes, float scale, int num_seqs, int num_heads,
                           int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                           int max_context_len, int partition_size, void* workspace,
                           size_t workspace_bytes, int dtype, void* stream)
{
    return attention_impl(out, q, k_cache, v_cache, block_tables, context_lens, alibi_slopes, scale, num_seqs,
                          num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_context_len,
                          partition_size, workspace, workspace_bytes, dtype, static_cast<hipStream_t>(stream),
                          nullptr);
}

int optgqa_paged_attention_static(void* out, const void* q, const void* k_cache, const void* v_cache,
                                  const int32_t* block_tables, const int32_t* context_lens,
                                  const float* alibi_slopes, float scale, int num_seqs, int num_heads,
                                  int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                                  int max_context_len, int dtype, void* stream)
{
    // the split the library would choose for these sizes must fit the static scratch: no silent
    // fall-back to the unsplit kernel here
    if (num_seqs > 0 && num_heads > 0 && num_kv_heads > 0 && head_dim > 0 && block_size > 0 &&
        max_context_len > 0 && num_heads % num_kv_heads == 0 && head_dim_ok(head_dim)) {
        const SplitPlan s = plan_split(num_seqs, num_heads, num_kv_heads, head_dim, block_size, max_context_len, 0);
        if (s.bytes > (size_t)OPTGQA_STATIC_SCRATCH_BYTES) return OPTGQA_ERR_WORKSPACE;
    }
    void* scratch = static_scratch();
    if (!scratch) return OPTGQA_ERR_LAUNCH;
    // Nothing in the scratch has to start at zero: every slot and plan entry the combine kernel
    // reads for a non-empty sequence is written by the streaming kernel of the same call.
    return attention_impl(out, q, k_cache, v_cache, block_tables, context_lens, alibi_slopes, scale, num_seqs,
                          num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_context_len, 0,
                          scratch, (size_t)OPTGQA_STATIC_SCRATCH_BYTES, dtype,
                          static_cast<hipStream_t>(stream), nullptr);
}

static int reshape_and_cache_fp8_impl(const void* k, const void* v, void* k_cache, void* v_cache,
                                      const int64_t* slot_mapping, int num_tokens, int num_kv_heads,
                                      int head_dim, int block_size, int64_t k_token_stride,
                                      int64_t v_token_stride, const KvScales& sc, int dtype, void* stream)
{
    if (num_tokens < 0 || num_kv_heads <= 0 || head_dim <= 0 || block_size <= 0) return OPTGQA_ERR_SHAPE;
    if (!dtype_ok(dtype) || !head_dim_ok(head_dim) || !block_size_ok(block_size)) return OPTGQA_ERR_UNSUPPORTED;
    const int64_t row = (int64_t)num_kv_heads * head_dim;
    if (k_token_stride < row || v_token_stride < row) return OPTGQA_ERR_SHAPE;
    if (sc.per_head() && !sc.v_heads) return OPTGQA_ERR_NULL;
    if (!sc.valid()) return OPTGQA_ERR_SHAPE;
    if (num_tokens == 0) return OPTGQA_OK;
    if (!k || !v || !k_cache || !v_cache || !slot_mapping) return OPTGQA_ERR_NULL;
    // 16-byte pieces in, 8-byte pieces out
    if (!aligned16(k) || !aligned16(v) || k_token_stride % 8 || v_token_stride % 8 ||
        ((reinterpret_cast<uintptr_t>(k_cache) | reinterpret_cast<uintptr_t>(v_cache)) & 7u))
        return OPTGQA_ERR_UNSUPPORTED;
    const int64_t threads = (int64_t)num_tokens * num_kv_heads * (head_dim / 8) * 2;
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffLL) return OPTGQA_ERR_SHAPE;
    // one fp32 division each (per KV head: the same division, in the kernel)
    const float k_inv = sc.per_head() ? 1.f : 1.0f / sc.k, v_inv = sc.per_head() ? 1.f : 1.0f / sc.v;
    hipStream_t st = static_cast<hipStream_t>(stream);
    auto kk = static_cast<const uint16_t*>(k);
    auto vv = static_cast<const uint16_t*>(v);
    auto kc = static_cast<unsigned char*>(k_cache);
    auto vc = static_cast<unsigned char*>(v_cache);
    return launch(dtype == OPTGQA_F16 ? reshape_and_cache_e4m3_kernel<kF16> : reshape_and_cache_e4m3_kernel<kBF16>,
                  dim3((unsigned)blocks), dim3(256), 0, st, kk, vv, kc, vc, slot_mapping, num_tokens, num_kv_heads,
                  head_dim, block_size, k_token_stride, v_token_stride, k_inv, v_inv, sc.k_heads, sc.v_heads);
}

int optgqa_reshape_and_cache_fp8(const void* k, const void* v, void* k_cache, void* v_cache,
                                 const int64_t* slot_mapping, int num_tokens, int num_kv_heads,
                                 int head_dim, int block_size, int64_t k_token_stride,
                                 int64_t v_token_stride, float k_scale, float v_scale,
                                 int dtype, void* stream)
{
    return reshape_and_cache_fp8_impl(k, v, k_cache, v_cache, slot_mapping, num_tokens, num_kv_heads, head_dim,
                                      block_size, k_token_stride, v_token_stride,
                                      KvScales{k_scale, v_scale, nullptr, nullptr}, dtype, stream);
}

int optgqa_reshape_and_cache_fp8_heads(const void* k, const void* v, void* k_cache, void* v_cache,
                                       const int64_t* slot_mapping, int num_tokens, int num_kv_heads,
                                       int head_dim, int block_size, int64_t k_token_stride,
                                       int64_t v_token_stride, const float* k_scales, const float* v_scales,
                                       int dtype, void* stream)
{
    if (!k_scales || !v_scales) return OPTGQA_ERR_NULL;
    return reshape_and_cache_fp8_impl(k, v, k_cache, v_cache, slot_mapping, num_tokens, num_kv_heads, head_dim,
                                      block_size, k_token_stride, v_token_stride,
                                      KvScales{1.f, 1.f, k_scales, v_scales}, dtype, stream);
}

int optgqa_paged_attention_fp8(void* out, const void* q, const void* k_cache, const void* v_cache,
                               const int32_t* block_tables, const int32_t* context_lens,
                               const float* alibi_slopes, float scale, float k_scale, float v_scale,
                               int num_seqs, int num_heads, int num_kv_heads, int head_dim,
                               int block_size, int max_blocks_per_seq, int max_context_len,
                               void* workspace, size_t workspace_bytes, int dtype, void* stream)
{
    const KvScales kv_scales{k_scale, v_scale, nullptr, nullptr};
    return attention_impl(out, q, k_cache, v_cache, block_tables, context_lens, alibi_slopes, scale, num_seqs,
                          num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_context_len,
                          OPTGQA_SPLIT_BALANCED, workspace, workspace_bytes, dtype,
                          static_cast<hipStream_t>(stream), nullptr, &kv_scales);
}

int optgqa_paged_attention_fp8_heads(void* out, const void* q, const void* k_cache, const void* v_cache,
                                     const int32_t* block_tables, const int32_t* context_lens,
                                     const float* alibi_slopes, float scale, const float* k_scales,
                                     const float* v_scales, int num_seqs, int num_heads, int num_kv_heads,
                                     int head_dim, int block_size, int max_blocks_per_seq, int max_context_len,
                                     void* workspace, size_t workspace_bytes, int dtype, void* stream)
{
    if (!k_scales || !v_scales) return OPTGQA_ERR_NULL;
    const KvScales kv_scales{1.f, 1.f, k_scales, v_scales};
    return attention_impl(out, q, k_cache, v_cache, block_tables, context_lens, alibi_slopes, scale, num_seqs,
                          num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_context_len,
                          OPTGQA_SPLIT_BALANCED, workspace, workspace_bytes, dtype,
                          static_cast<hipStream_t>(stream), nullptr, &kv_scales);
}

int optgqa_decode_step(void* out, const void* q, const void* k_new, const void* v_new, void* k_cache,
                       void* v_cache, const int32_t* block_tables, const int32_t* context_lens,
                       const float* alibi_slopes, float scale, int num_seqs, int num_heads,
                       int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                       int max_context_len, int64_t k_token_stride, int64_t v_token_stride,
                       void* workspace, size_t workspace_bytes, int dtype, void* stream)
{
    const StepInputs step{k_new, v_new, k_token_stride, v_token_stride, k_cache, v_cache};
    return attention_impl(out, q, k_cache, v_cache, block_tables, context_lens, alibi_slopes, scale, num_seqs,
                          num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_context_len, 0,
                          workspace, workspace_bytes, dtype, static_cast<hipStream_t>(stream), &step);
}

int optgqa_paged_attention_window(void* out, const void* q, const void* k_cache, const void* v_cache,
                                  const int32_t* block_tables, const int32_t* context_lens,
                                  const float* alibi_slopes, float scale, int window, int num_seqs,
                                  int num_heads, int num_kv_heads, int head_dim, int block_size,
                                  int max_blocks_per_seq, int max_context_len, void* workspace,
                                  size_t workspace_bytes, int dtype, void* stream)
{
    if (window <= 0) return OPTGQA_ERR_SHAPE;
    return attention_impl(out, q, k_cache, v_cache, block_tables, context_lens, alibi_slopes, scale, num_seqs,
                          num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_context_len,
                          OPTGQA_SPLIT_BALANCED, workspace, workspace_bytes, dtype,
                          static_cast<hipStream_t>(stream), nullptr, nullptr, window);
}

int optgqa_decode_step_window(void* out, const void* q, const void* k_new, const void* v_new, void* k_cache,
                              void* v_cache, const int32_t* block_tables, const int32_t* context_lens,
                              const float* alibi_slopes, float scale, int window, int num_seqs,
                              int num_heads, int num_kv_heads, int head_dim, int block_size,
                              int max_blocks_per_seq, int max_context_len, int64_t k_token_stride,
                              int64_t v_token_stride, void* workspace, size_t workspace_bytes,
                              int dtype, void* stream)
{
    if (window <= 0) return OPTGQA_ERR_SHAPE;
    const StepInputs step{k_new, v_new, k_token_stride, v_token_stride, k_cache, v_cache};
    return attention_impl(out, q, k_cache, v_cache, block_tables, context_lens, alibi_slopes, scale, num_seqs,
                          num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_context_len,
                          OPTGQA_SPLIT_BALANCED, workspace, workspace_bytes, dtype,
                          static_cast<hipStream_t>(stream), &step, nullptr, window);
}

int optgqa_decode_step_fp8(void* out, const void* q, const void* k_new, const void* v_new, void* k_cache,
                           void* v_cache, const int32_t* block_tables, const int32_t* context_lens,
                           const float* alibi_slopes, float scale, float k_scale, float v_scale,
                           int num_seqs, int num_heads, int num_kv_heads, int head_dim, int block_size,
                           int max_blocks_per_seq, int max_context_len, int64_t k_token_stride,
                           int64_t v_token_stride, void* workspace, size_t workspace_bytes,
                           int dtype, void* stream)
{
    const StepInputs step{k_new, v_new, k_token_stride, v_token_stride, k_cache, v_cache};
    const KvScales kv_scales{k_scale, v_scale, nullptr, nullptr};
    return attention_impl(out, q, k_cache, v_cache, block_tables, context_lens, alibi_slopes, scale, num_seqs,
                          num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_context_len,
                          OPTGQA_SPLIT_BALANCED, workspace, workspace_bytes, dtype,
                          static_cast<hipStream_t>(stream), &step, &kv_scales);
}

int optgqa_decode_step_fp8_heads(void* out, const void* q, const void* k_new, const void* v_new, void* k_cache,
                                 void* v_cache, const int32_t* block_tables, const int32_t* context_lens,
                                 const float* alibi_slopes, float scale, const float* k_scales,
                                 const float* v_scales, int num_seqs, int num_heads, int num_kv_heads,
                                 int head_dim, int block_size, int max_blocks_per_seq, int max_context_len,
                                 int64_t k_token_stride, int64_t v_token_stride, void* workspace,
                                 size_t workspace_bytes, int dtype, void* stream)
{
    if (!k_scales || !v_scales) return OPTGQA_ERR_NULL;
    const StepInputs step{k_new, v_new, k_token_stride, v_token_stride, k_cache, v_cache};
    const KvScales kv_scales{1.f, 1.f, k_scales, v_scales};
    return attention_impl(out, q, k_cache, v_cache, block_tables, context_lens, alibi_slopes, scale, num_seqs,
                          num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_context_len,
                          OPTGQA_SPLIT_BALANCED, workspace, workspace_bytes, dtype,
                          static_cast<hipStream_t>(stream), &step, &kv_scales);
}

int optgqa_shared_prefix_bundle(int num_heads, int num_kv_heads, int head_dim)
{
    if (num_heads <= 0 || num_kv_heads <= 0 || num_heads % num_kv_heads) return OPTGQA_ERR_SHAPE;
    if (!head_dim_ok(head_dim)) return OPTGQA_ERR_UNSUPPORTED;
    return kMmaMaxHeads / mfma_heads_per_workgroup(num_heads / num_kv_heads);
}

size_t optgqa_shared_prefix_workspace_bytes(int num_seqs, int num_heads, int num_kv_heads, int head_dim,
                                            int block_size, int max_context_len)
{
    if (num_seqs <= 0 || num_heads <= 0 || num_kv_heads <= 0 || !head_dim_ok(head_dim) || block_size <= 0 ||
        max_context_len <= 0 || num_heads % num_kv_heads)
        return 0;
    const SplitPlan s = plan_split(num_seqs, num_heads, num_kv_heads, head_dim, block_size, max_context_len,
                                   OPTGQA_SPLIT_BALANCED, 0, true);
    return s.partition_size == OPTGQA_SPLIT_BALANCED ? s.bytes : 0;
}

int optgqa_paged_attention_shared(void* out, const void* q, const void* k_cache, const void* v_cache,
                                  const int32_t* block_tables, const int32_t* context_lens,
                                  const int32_t* shared_blocks, const float* alibi_slopes, float scale,
                                  int num_seqs, int num_heads, int num_kv_heads, int head_dim, int block_size,
                                  int max_blocks_per_seq, int max_context_len, void* workspace,
                                  size_t workspace_bytes, int dtype, void* stream)
{
    if (!shared_blocks && num_seqs > 0) return OPTGQA_ERR_NULL;
    return attention_impl(out, q, k_cache, v_cache, block_tables, context_lens, alibi_slopes, scale, num_seqs,
                          num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_context_len,
                          OPTGQA_SPLIT_BALANCED, workspace, workspace_bytes, dtype,
                          static_cast<hipStream_t>(stream), nullptr, nullptr, 0, shared_blocks);
}

int optgqa_decode_step_shared(void* out, const void* q, const void* k_new, const void* v_new, void* k_cache,
                              void* v_cache, const int32_t* block_tables, const int32_t* context_lens,
                              const int32_t* shared_blocks, const float* alibi_slopes, float scale, int num_seqs,
                              int num_heads, int num_kv_heads, int head_dim, int block_size,
                              int max_blocks_per_seq, int max_context_len, int64_t k_token_stride,
                              int64_t v_token_stride, void* workspace, size_t workspace_bytes,
                              int dtype, void* stream)
{
    if (!shared_blocks && num_seqs > 0) return OPTGQA_ERR_NULL;
    const StepInputs step{k_new, v_new, k_token_stride, v_token_stride, k_cache, v_cache};
    return attention_impl(out, q, k_cache, v_cache, block_tables, context_lens, alibi_slopes, scale, num_seqs,
                          num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_context_len,
                          OPTGQA_SPLIT_BALANCED, workspace, workspace_bytes, dtype,
                          static_cast<hipStream_t>(stream), &step, nullptr, 0, shared_blocks);
}

int optgqa_validate_shared_prefix_host(const int32_t* block_tables_host, const int32_t* context_lens_host,
                                       const int32_t* shared_blocks_host, int num_seqs, int max_blocks_per_seq,
                                       int block_size, int bundle, int new_tokens)
{
    if (num_seqs < 0 || max_blocks_per_seq <= 0 || block_size <= 0 || bundle <= 0 || new_tokens < 0)
        return OPTGQA_ERR_SHAPE;
    if (num_seqs == 0) return OPTGQA_OK;
    if (!block_tables_host || !context_lens_host || !shared_blocks_host) return OPTGQA_ERR_NULL;
    for (int b = 0; b < num_seqs; ++b) {
        const int s = shared_blocks_host[b];
        if (s < 0) return OPTGQA_ERR_TABLE;
        if (s == 0) continue;
        const int b0 = b - b % bundle;
        if (b == b0) return OPTGQA_ERR_TABLE;                   // a leader shares with nobody before it
        // whole blocks that both the sequence and its leader already hold in the cache
        const int64_t cached = (int64_t)context_lens_host[b] - new_tokens, cached0 = (int64_t)context_lens_host[b0] - new_tokens;
        if ((int64_t)s * block_size > cached || (int64_t)s * block_size > cached0 || s > max_blocks_per_seq)
            return OPTGQA_ERR_TABLE;
        for (int i = 0; i < s; ++i)
            if (block_tables_host[(int64_t)b * max_blocks_per_seq + i] != block_tables_host[(int64_t)b0 * max_blocks_per_seq + i])
                return OPTGQA_ERR_TABLE;
    }
    return OPTGQA_OK;
}

static int prefill_impl(void* out, const void* q, const void* k_cache, const void* v_cache,
                        const int32_t* block_tables, const int32_t* context_lens,
                        const int32_t* cu_q_lens, const float* alibi_slopes, float scale,
                        int num_seqs, int num_heads, int num_kv_heads, int head_dim, int block_size,
                        int max_blocks_per_seq, int max_q_len, int dtype, void* stream,
                        const KvScales* kv_scales, int window = 0)
{
    if (kv_scales && kv_scales->per_head() && !kv_scales->v_heads) return OPTGQA_ERR_NULL;
    if (kv_scales && !kv_scales->valid()) return OPTGQA_ERR_SHAPE;
    if (num_seqs < 0 || num_heads <= 0 || num_kv_heads <= 0 || head_dim <= 0 || block_size <= 0 ||
        max_blocks_per_seq <= 0 || max_q_len < 0)
        return OPTGQA_ERR_SHAPE;
    if (!std::isfinite(scale)) return OPTGQA_ERR_SHAPE;
    if (num_heads % num_kv_heads) return OPTGQA_ERR_SHAPE;
    if (!dtype_ok(dtype) || !head_dim_ok(head_dim) || !block_size_ok(block_size)) return OPTGQA_ERR_UNSUPPORTED;
    if (num_seqs == 0 || max_q_len == 0) return OPTGQA_OK;
    if (!out || !q || !k_cache || !v_cache || !block_tables || !context_lens || !cu_q_lens) return OPTGQA_ERR_NULL;
    if (!aligned16(out) || !aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache)) return OPTGQA_ERR_UNSUPPORTED;
    if (num_seqs > 65535) return OPTGQA_ERR_SHAPE;
    PrefillParams p;
    p.out = out;
    p.q = q;
    p.k_cache = k_cache;
    p.v_cache = v_cache;
    p.block_tables = block_tables;
    p.context_lens = context_lens;
    p.cu_q_lens = cu_q_lens;
    p.slopes = alibi_slopes;
    const bool heads = kv_scales && kv_scales->per_head();
    p.scale2 = prefill_scale2(scale * (kv_scales && !heads ? kv_scales->k : 1.f));
    p.out_scale = kv_scales && !heads ? kv_scales->v : 1.f;
    p.k_scales = heads ? kv_scales->k_heads : nullptr;
    p.v_scales = heads ? kv_scales->v_heads : nullptr;
    p.window = window > 0 ? window : 0;
    p.k_in = p.v_in = nullptr;
    p.k_in_stride = p.v_in_stride = 0;
    p.k_cache_w = p.v_cache_w = nullptr;
    p.num_heads = num_heads;
    p.num_kv_heads = num_kv_heads;
    p.block_size = block_size;
    p.max_blocks_per_seq = max_blocks_per_seq;
    return launch_prefill(p, num_seqs, max_q_len, head_dim, dtype, static_cast<hipStream_t>(stream), kv_scales != nullptr);
}

int optgqa_paged_prefill(void* out, const void* q, const void* k_cache, const void* v_cache,
                         const int32_t* block_tables, const int32_t* context_lens,
                         const int32_t* cu_q_lens, const float* alibi_slopes, float scale,
                         int num_seqs, int num_heads, int num_kv_heads, int head_dim, int block_size,
                         int max_blocks_per_seq, int max_q_len, int dtype, void* stream)
{
    return prefill_impl(out, q, k_cache, v_cache, block_tables, context_lens, cu_q_lens, alibi_slopes, scale,
                        num_seqs, num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_q_len,
                        dtype, stream, nullptr);
}

int optgqa_paged_prefill_fp8(void* out, const void* q, const void* k_cache, const void* v_cache,
                             const int32_t* block_tables, const int32_t* context_lens,
                             const int32_t* cu_q_lens, const float* alibi_slopes, float scale,
                             float k_scale, float v_scale, int num_seqs, int num_heads,
                             int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                             int max_q_len, int dtype, void* stream)
{
    const KvScales kv_scales{k_scale, v_scale, nullptr, nullptr};
    return prefill_impl(out, q, k_cache, v_cache, block_tables, context_lens, cu_q_lens, alibi_slopes, scale,
                        num_seqs, num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_q_len,
                        dtype, stream, &kv_scales);
}

int optgqa_paged_prefill_fp8_heads(void* out, const void* q, const void* k_cache, const void* v_cache,
                                   const int32_t* block_tables, const int32_t* context_lens,
                                   const int32_t* cu_q_lens, const float* alibi_slopes, float scale,
                                   const float* k_scales, const float* v_scales, int num_seqs, int num_heads,
                                   int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                                   int max_q_len, int dtype, void* stream)
{
    if (!k_scales || !v_scales) return OPTGQA_ERR_NULL;
    const KvScales kv_scales{1.f, 1.f, k_scales, v_scales};
    return prefill_impl(out, q, k_cache, v_cache, block_tables, context_lens, cu_q_lens, alibi_slopes, scale,
                        num_seqs, num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_q_len,
                        dtype, stream, &kv_scales);
}

int optgqa_paged_prefill_window(void* out, const void* q, const void* k_cache, const void* v_cache,
                                const int32_t* block_tables, const int32_t* context_lens,
                                const int32_t* cu_q_lens, const float* alibi_slopes, float scale,
                                int window, int num_seqs, int num_heads, int num_kv_heads, int head_dim,
                                int block_size, int max_blocks_per_seq, int max_q_len, int dtype,
                                void* stream)
{
    if (window <= 0) return OPTGQA_ERR_SHAPE;
    return prefill_impl(out, q, k_cache, v_cache, block_tables, context_lens, cu_q_lens, alibi_slopes, scale,
                        num_seqs, num_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, max_q_len,
                        dtype, stream, nullptr, window);
}

int optgqa_prompt_prefill(void* out, const void* q, const void* k, const void* v, void* k_cache, void* v_cache,
                          const int32_t* block_tables, const int32_t* cu_seq_lens, const float* alibi_slopes,
                          float scale, int num_seqs, int num_heads, int num_kv_heads, int head_dim,
                          int block_size, int max_blocks_per_seq, int max_seq_len, int64_t k_token_stride,
                          int64_t v_token_stride, int dtype, void* stream)
{
    if (num_seqs < 0 || num_heads <= 0 || num_kv_heads <= 0 || head_dim <= 0 || max_seq_len < 0)
        return OPTGQA_ERR_SHAPE;
    if (!std::isfinite(scale)) return OPTGQA_ERR_SHAPE;
    if (num_heads % num_kv_heads) return OPTGQA_ERR_SHAPE;
    const int64_t row = (int64_t)num_kv_heads * head_dim;
    // (the kernel forms byte offsets between token rows in 32 bits)
    if (k_token_stride < row || v_token_stride < row || k_token_stride > (1LL << 30) || v_token_stride > (1LL << 30))
        return OPTGQA_ERR_SHAPE;
    if ((k_cache == nullptr) != (v_cache == nullptr)) return OPTGQA_ERR_NULL;
    const bool store = k_cache != nullptr;
    if (store) {
        if (block_size <= 0 || max_blocks_per_seq <= 0) return OPTGQA_ERR_SHAPE;
        if ((int64_t)max_seq_len > (int64_t)max_blocks_per_seq * block_size) return OPTGQA_ERR_SHAPE;
        if (!block_size_ok(block_size)) return OPTGQA_ERR_UNSUPPORTED;
    }
    if (!dtype_ok(dtype) || !head_dim_ok(head_dim)) return OPTGQA_ERR_UNSUPPORTED;
    if (k_token_stride % 8 || v_token_stride % 8) return OPTGQA_ERR_UNSUPPORTED;   // rows move as 16-byte pieces
    if (num_seqs == 0 || max_seq_len == 0) return OPTGQA_OK;
    if (!out || !q || !k || !v || !cu_seq_lens || (store && !block_tables)) return OPTGQA_ERR_NULL;
    if (!aligned16(out) || !aligned16(q) || !aligned16(k) || !aligned16(v) ||
        (store && (!aligned16(k_cache) || !aligned16(v_cache))))
        return OPTGQA_ERR_UNSUPPORTED;
    if (num_seqs > 65535) return OPTGQA_ERR_SHAPE;
    PrefillParams p;
    p.out = out;
    p.q = q;
    p.k_cache = p.v_cache = nullptr;
    p.block_tables = block_tables;
    p.context_lens = nullptr;
    p.cu_q_lens = cu_seq_lens;
    p.slopes = alibi_slopes;
    p.scale2 = prefill_scale2(scale);
    p.out_scale = 1.f;
    p.k_scales = p.v_scales = nullptr;
    p.window = 0;
    p.k_in = k;
    p.v_in = v;
    p.k_in_stride = k_token_stride;
    p.v_in_stride = v_token_stride;
    p.k_cache_w = k_cache;
    p.v_cache_w = v_cache;
    p.num_heads = num_heads;
    p.num_kv_heads = num_kv_heads;
    p.block_size = store ? block_size : 16;
    p.max_blocks_per_seq = store ? max_blocks_per_seq : 0;
    return launch_prefill(p, num_seqs, max_seq_len, head_dim, dtype, static_cast<hipStream_t>(stream), false, true);
}

int optgqa_prefill_step(void* out, const void* q, const void* k_new, const void* v_new, void* k_cache,
                        void* v_cache, const int32_t* block_tables, const int32_t* context_lens,
                        const int32_t* cu_q_lens, const float* alibi_slopes, float scale, int num_seqs,
                        int num_heads, int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                        int max_q_len, int64_t k_token_stride, int64_t v_token_stride, int dtype, void* stream)
{
    if (num_seqs < 0 || num_heads <= 0 || num_kv_heads <= 0 || head_dim <= 0 || block_size <= 0 ||
        max_blocks_per_seq <= 0 || max_q_len < 0)
        return OPTGQA_ERR_SHAPE;
    if (!std::isfinite(scale)) return OPTGQA_ERR_SHAPE;
    if (num_heads % num_kv_heads) return OPTGQA_ERR_SHAPE;
    const int64_t row = (int64_t)num_kv_heads * head_dim;
    // (the kernel forms byte offsets between token rows in 32 bits)
    if (k_token_stride < row || v_token_stride < row || k_token_stride > (1LL << 30) || v_token_stride > (1LL << 30))
        return OPTGQA_ERR_SHAPE;
    if (!dtype_ok(dtype) || !head_dim_ok(head_dim) || !block_size_ok(block_size)) return OPTGQA_ERR_UNSUPPORTED;
    if (k_token_stride % 8 || v_token_stride % 8) return OPTGQA_ERR_UNSUPPORTED;   // rows move as 16-byte pieces
    if (num_seqs == 0 || max_q_len == 0) return OPTGQA_OK;
    if (!out || !q || !k_new || !v_new || !k_cache || !v_cache || !block_tables || !context_lens || !cu_q_lens)
        return OPTGQA_ERR_NULL;
    if (!aligned16(out) || !aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) ||
        !aligned16(v_cache))
        return OPTGQA_ERR_UNSUPPORTED;
    if (num_seqs > 65535) return OPTGQA_ERR_SHAPE;
    PrefillParams p;
    p.out = out;
    p.q = q;
    p.k_cache = k_cache;
    p.v_cache = v_cache;
    p.block_tables = block_tables;
    p.context_lens = context_lens;
    p.cu_q_lens = cu_q_lens;
    p.slopes = alibi_slopes;
    p.scale2 = prefill_scale2(scale);
    p.out_scale = 1.f;
    p.k_scales = p.v_scales = nullptr;
    p.window = 0;
    p.k_in = k_new;
    p.v_in = v_new;
    p.k_in_stride = k_token_stride;
    p.v_in_stride = v_token_stride;
    p.k_cache_w = k_cache;
    p.v_cache_w = v_cache;
    p.num_heads = num_heads;
    p.num_kv_heads = num_kv_heads;
    p.block_size = block_size;
    p.max_blocks_per_seq = max_blocks_per_seq;
    return launch_prefill(p, num_seqs, max_q_len, head_dim, dtype, static_cast<hipStream_t>(stream), false, false, true);
}

int optgqa_stream_probe(const void* k_pool, const void* v_pool, size_t pool_bytes,
                        const int32_t* tile_list, const int32_t* tile_list_host, int num_workgroups,
                        int tiles_per_wave, void* sink, void* stream)
{
    if (num_workgroups <= 0 || tiles_per_wave <= 0 || pool_bytes < 4096) return OPTGQA_ERR_SHAPE;
    if (!k_pool || !v_pool || !tile_list || !tile_list_host || !sink) return OPTGQA_ERR_NULL;
    if (!aligned16(k_pool) || !aligned16(v_pool) || !aligned16(sink)) return OPTGQA_ERR_UNSUPPORTED;
    // every listed piece must lie inside the pools: checked here, on the host copy of the list
    const int64_t pieces = (int64_t)(pool_bytes / 4096);
    const int64_t n = (int64_t)num_workgroups * 4 * tiles_per_wave;
    for (int64_t i = 0; i < n; ++i)
        if (tile_list_host[i] < 0 || tile_list_host[i] >= pieces) return OPTGQA_ERR_TABLE;
    return launch(stream_probe_kernel, dim3(num_workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                  static_cast<const unsigned char*>(k_pool), static_cast<const unsigned char*>(v_pool), tile_list,
                  tiles_per_wave, static_cast<uint4*>(sink));
}

int optgqa_gather_kv(void* k_out, void* v_out, const void* k_cache, const void* v_cache,
                     const int32_t* block_tables, const int32_t* context_lens, int num_seqs,
                     int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                     int max_context_len, int dtype, void* stream)
{
    if (num_seqs < 0 || num_kv_heads <= 0 || head_dim <= 0 || block_size <= 0 || max_blocks_per_seq <= 0 ||
        max_context_len < 0)
        return OPTGQA_ERR_SHAPE;
    if (!dtype_ok(dtype) || !head_dim_ok(head_dim) || !block_size_ok(block_size)) return OPTGQA_ERR_UNSUPPORTED;
    if (num_seqs == 0 || max_context_len == 0) return OPTGQA_OK;
    if (!k_out || !v_out || !k_cache || !v_cache || !block_tables || !context_lens) return OPTGQA_ERR_NULL;
    if (!aligned16(k_out) || !aligned16(v_out) || !aligned16(k_cache) || !aligned16(v_cache)) return OPTGQA_ERR_UNSUPPORTED;
    if (num_seqs > 65535) return OPTGQA_ERR_SHAPE;
    const int64_t pieces = (int64_t)max_context_len * num_kv_heads * (head_dim / 8);
    const dim3 grid((unsigned)((pieces + 255) / 256), num_seqs, 2);
    return launch(gather_kv_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream),
                  static_cast<uint16_t*>(k_out), static_cast<uint16_t*>(v_out), static_cast<const uint16_t*>(k_cache),
                  static_cast<const uint16_t*>(v_cache), block_tables, context_lens, num_kv_heads, head_dim,
                  block_size, max_blocks_per_seq, max_context_len);
}

int optgqa_validate_tables_host(const int32_t* block_tables_host, const int32_t* context_lens_host,
                                int num_seqs, int max_blocks_per_seq, int block_size, int num_blocks)
{
    if (num_seqs < 0 || max_blocks_per_seq <= 0 || block_size <= 0 || num_blocks <= 0) return OPTGQA_ERR_SHAPE;
    if (num_seqs == 0) return OPTGQA_OK;
    if (!block_tables_host || !context_lens_host) return OPTGQA_ERR_NULL;
    for (int b = 0; b < num_seqs; ++b) {
        const int L = context_lens_host[b];
        if (L < 0 || (int64_t)L > (int64_t)max_blocks_per_seq * block_size) return OPTGQA_ERR_TABLE;
        const int nb = (L + block_size - 1) / block_size;
        for (int i = 0; i < nb; ++i) {
            const int id = block_tables_host[(int64_t)b * max_blocks_per_seq + i];
            if (id < 0 || id >= num_blocks) return OPTGQA_ERR_TABLE;
        }
    }
    return OPTGQA_OK;
}

}  // extern "C"
