// Host side of the C ABI declared in include/gbnn.h: argument checks and kernel dispatch.
#include <atomic>

#include "gbnn_device.h"
#include "gbnn_internal.h"

using namespace gbnn;

// The prepared table of gbnn_retrieve_static: device memory of the library itself, one copy on every
// GPU the library runs on, held until the process ends.  Room for the table of any network of up to
// GBNN_STATIC_MAX_N neurons ((n + C + 2) rows of n/32 words, rounded up to 256 bytes, plus 256 for the
// flags).  In host code this name only stands for the symbol; the array's address on a device comes
// from hipGetSymbolAddress (static_scratch below).
constexpr size_t kStaticScratchBytes =
    ((size_t)(GBNN_STATIC_MAX_N + GBNN_MAX_C + 2) * (GBNN_STATIC_MAX_N / 32) * 4 + 255) / 256 * 256 + 256 +
    (size_t)GBNN_MAX_C * (GBNN_STATIC_MAX_N / 32) * 4;  // (+ the canonical summaries of a padded network)
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// Address of `scratch` on the current device, looked up once per device (with that device current).
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];
void *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // (two threads racing here store the same address)
    }
    return p;
}

bool shape_ok(int C, int L)
{
    if (C < 2 || C > GBNN_MAX_C || L < 1) return false;
    const int64_t n = (int64_t)C * (int64_t)L;
    return n <= GBNN_MAX_N;
}

bool rule_ok(int rule) { return rule == GBNN_SUM_OF_SUM || rule == GBNN_SUM_OF_MAX || rule == GBNN_HYBRID; }

bool aligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// What gbnn_set_kernel_choice last set (tests and A/B timing); both start as "the library chooses".
std::atomic<int> g_retrieve_family{GBNN_FAMILY_AUTO};
std::atomic<int> g_store_kernel{GBNN_STORE_AUTO};

// Kernel family for a call: 0 = any-shape kernel; 1, 2, 4, 8 = one wavefront per probe with that many packed
// words per lane; kHalfPath = half a wavefront per probe.
constexpr int kHalfPath = 10;
int pick_path(int C, int L, int rule, const void *V0, const void *Vout)
{
    const int family = g_retrieve_family.load(std::memory_order_relaxed);
    if (family == GBNN_FAMILY_GENERIC) return 0;
    (void)V0;
    (void)Vout;  // (any alignment: the kernels load and store the activity in pieces of 16, 4 or 1 bytes)
    if (family != GBNN_FAMILY_WAVE && half_wave_serves(C, L)) return kHalfPath;
    (void)rule;
    return wave_words_per_lane(C, L);
}

// Checks common to both boundaries, then the launch.
int retrieve_common(RetrieveArgs &a, const uint32_t *W, int C, int L, int64_t K, int rule, int gamma, int max_iters,
                    int32_t *iters_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < workspace_total_bytes(C, L)) return GBNN_ERR_WORKSPACE;
    if (K == 0) return GBNN_OK;
    const Geometry g = geometry(C, L);
    const char *ws = static_cast<const char *>(workspace);
    a.W = W;
    a.nw = (C * L + 31) / 32;
    a.Lp = g.Lp;
    a.np = g.np;
    a.nwp = g.nwp;
    a.Wb = reinterpret_cast<const uint32_t *>(ws);
    a.has = reinterpret_cast<const uint32_t *>(ws + workspace_has_offset(C, L));
    a.hasc = g.padded ? reinterpret_cast<const uint32_t *>(ws + workspace_canonical_offset(C, L)) : a.has;
    a.full = reinterpret_cast<const uint64_t *>(ws + workspace_full_offset(C, L));
    a.aligned16 = L % 16 == 0 && aligned(a.V0, 16) && aligned(a.Vout, 16);
    // Probes that cannot stay in the 256 MB memory-side cache from one call to the next anyway are read with
    // non-temporal loads where the table is larger than one of the 4 MiB L2s: the table then keeps more of the
    // L2 (16x512, K=131072: 402 -> 388 us).  A batch that fits the memory-side cache is read faster without
    // (8x256, K=65536: 42 us against 53 us).
    a.stream_in = a.V0 && (int64_t)K * C * L >= (512ll << 20) && workspace_has_offset(C, L) > ((size_t)4 << 20);
    a.iters = iters_out;
    a.K = K;
    a.C = C;
    a.L = L;
    a.n = C * L;
    a.rule = rule;
    a.gamma = gamma;
    a.max_iters = max_iters;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int path = pick_path(C, L, rule, a.V0, a.Vout);
    const hipError_t e = path == kHalfPath ? launch_retrieve_half(a, s)
                         : path            ? launch_retrieve_wave(a, path, s)
                                           : launch_retrieve_generic(a, s);
    return e == hipSuccess ? GBNN_OK : GBNN_ERR_DEVICE;
}

}  // namespace

namespace gbnn {
namespace {
// The reference copy of the benchmark: every wavefront moves 2 KiB, lane l the 16 bytes at 16 l of each KiB.
template <bool STREAMING>
__global__ __launch_bounds__(256) void k_reference_copy(const uint8_t *src, uint8_t *dst, size_t bytes)
{
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const size_t at = wave * 2048 + 16 * (threadIdx.x & 63);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const size_t o = at + 1024 * h;
        if (o < bytes) {
            if (STREAMING)
                store16_nontemporal(dst + o, load16_nontemporal(src + o));
            else
                *reinterpret_cast<uint4 *>(dst + o) = *reinterpret_cast<const uint4 *>(src + o);
        }
    }
}
}  // namespace
}  // namespace gbnn

extern "C" {

size_t gbnn_w_row_words(int C, int L)
{
    if (!shape_ok(C, L)) return 0;
    return (size_t)((C * L + 31) / 32);
}

size_t gbnn_w_bytes(int C, int L)
{
    if (!shape_ok(C, L)) return 0;
    return (size_t)C * (size_t)L * gbnn_w_row_words(C, L) * sizeof(uint32_t);
}

size_t gbnn_workspace_bytes(int C, int L, int64_t K, int rule)
{
    if (!shape_ok(C, L) || K < 0 || K > GBNN_MAX_K || !rule_ok(rule)) return 0;
    return workspace_total_bytes(C, L);
}

int gbnn_store(uint32_t *W, int C, int L, const int32_t *msgs, int64_t M, int32_t *status, void *stream)
{
    if (!shape_ok(C, L) || M < 0) return GBNN_ERR_SHAPE;
    if (!W || (M > 0 && !msgs)) return GBNN_ERR_NULL;
    const int choice = g_store_kernel.load(std::memory_order_relaxed);
    const int path = choice == GBNN_STORE_ATOMIC ? kStoreAtomic : choice == GBNN_STORE_ROWS ? kStoreRows : kStoreAuto;
    const hipError_t e = launch_store(W, C, L, (int)gbnn_w_row_words(C, L), msgs, M, status, path,
                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GBNN_OK : GBNN_ERR_DEVICE;
}

int gbnn_prepare(const uint32_t *W, int C, int L, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!shape_ok(C, L)) return GBNN_ERR_SHAPE;
    if (!W) return GBNN_ERR_NULL;
    const int nw = (int)gbnn_w_row_words(C, L);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < workspace_total_bytes(C, L)) return GBNN_ERR_WORKSPACE;
    const hipError_t e = launch_prepare(W, C, L, nw, static_cast<char *>(workspace), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GBNN_OK : GBNN_ERR_DEVICE;
}

int gbnn_store_update(uint32_t *W, int C, int L, const int32_t *msgs, int64_t M, int32_t *status, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    if (!shape_ok(C, L) || M < 0) return GBNN_ERR_SHAPE;
    if (!W || (M > 0 && !msgs)) return GBNN_ERR_NULL;
    const int nw = (int)gbnn_w_row_words(C, L);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < workspace_total_bytes(C, L)) return GBNN_ERR_WORKSPACE;
    const hipError_t e = launch_store_update(W, C, L, nw, msgs, M, status, static_cast<char *>(workspace),
                                             static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GBNN_OK : GBNN_ERR_DEVICE;
}

int gbnn_retrieve(const uint32_t *W, int C, int L, const uint8_t *V0, uint8_t *V_out, int64_t K, int rule,
                  int gamma, int max_iters, int32_t *iters_out, void *workspace, size_t workspace_bytes,
                  void *stream)
{
    if (!shape_ok(C, L) || K < 0 || K > GBNN_MAX_K) return GBNN_ERR_SHAPE;
    if (!rule_ok(rule)) return GBNN_ERR_RULE;
    if (gamma < 0 || gamma > GBNN_MAX_GAMMA) return GBNN_ERR_GAMMA;
    if (max_iters < 1) return GBNN_ERR_ITERS;
    if (!W || (K > 0 && (!V0 || !V_out))) return GBNN_ERR_NULL;
    RetrieveArgs a{};
    a.V0 = V0;
    a.Vout = V_out;
    return retrieve_common(a, W, C, L, K, rule, gamma, max_iters, iters_out, workspace, workspace_bytes, stream);
}

int gbnn_retrieve_static(const uint32_t *W, int C, int L, const uint8_t *V0, uint8_t *V_out, int64_t K, int rule,
                         int gamma, int max_iters, int32_t *iters_out, void *stream)
{
    if (!shape_ok(C, L) || K < 0 || K > GBNN_MAX_K) return GBNN_ERR_SHAPE;
    if (!rule_ok(rule)) return GBNN_ERR_RULE;
    if (gamma < 0 || gamma > GBNN_MAX_GAMMA) return GBNN_ERR_GAMMA;
    if (max_iters < 1) return GBNN_ERR_ITERS;
    if (!W || (K > 0 && (!V0 || !V_out))) return GBNN_ERR_NULL;
    const int nw = (int)gbnn_w_row_words(C, L);
    (void)nw;
    if (C * L > GBNN_STATIC_MAX_N || workspace_total_bytes(C, L) > kStaticScratchBytes) return GBNN_ERR_TOO_LARGE;
    if (K == 0) return GBNN_OK;
    void *ws = static_scratch();
    if (!ws) return GBNN_ERR_DEVICE;
    // every word of the table that retrieval reads is rewritten here, so what the last call left does not matter
    const int e = gbnn_prepare(W, C, L, ws, kStaticScratchBytes, stream);
    if (e != GBNN_OK) return e;
    return gbnn_retrieve(W, C, L, V0, V_out, K, rule, gamma, max_iters, iters_out, ws, kStaticScratchBytes, stream);
}

int gbnn_retrieve_symbols(const uint32_t *W, int C, int L, const int32_t *probes, int64_t K, int rule, int gamma,
                          int max_iters, uint32_t *bits_out, int32_t *symbols_out, int32_t *iters_out,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    if (!shape_ok(C, L) || K < 0 || K > GBNN_MAX_K) return GBNN_ERR_SHAPE;
    if (!rule_ok(rule)) return GBNN_ERR_RULE;
    if (gamma < 0 || gamma > GBNN_MAX_GAMMA) return GBNN_ERR_GAMMA;
    if (max_iters < 1) return GBNN_ERR_ITERS;
    if (!W || (K > 0 && !probes)) return GBNN_ERR_NULL;
    RetrieveArgs a{};
    a.sym_in = probes;
    a.bits_out = bits_out;
    a.sym_out = symbols_out;
    return retrieve_common(a, W, C, L, K, rule, gamma, max_iters, iters_out, workspace, workspace_bytes, stream);
}

size_t gbnn_sparse_bytes(int C, int L, int64_t nnz)
{
    if (!shape_ok(C, L) || L % 32 != 0 || nnz < 0 || nnz > 0xFFFFFFFFll) return 0;
    const int n = C * L;
    return sparse_cols_offset(C, n, (int)gbnn_w_row_words(C, L)) + (((size_t)nnz * 2 + 255) & ~(size_t)255);
}

int gbnn_sparse_count(const uint32_t *W, int C, int L, uint64_t *nnz_out, void *stream)
{
    if (!shape_ok(C, L)) return GBNN_ERR_SHAPE;
    if (!W || !nnz_out) return GBNN_ERR_NULL;
    const hipError_t e = launch_sparse_count(W, C * L, (int)gbnn_w_row_words(C, L),
                                             reinterpret_cast<unsigned long long *>(nnz_out),
                                             static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GBNN_OK : GBNN_ERR_DEVICE;
}

int gbnn_sparsify(const uint32_t *W, int C, int L, void *Wp, size_t Wp_bytes, int32_t *status, void *stream)
{
    if (!shape_ok(C, L) || L % 32 != 0) return GBNN_ERR_SHAPE;
    if (!W) return GBNN_ERR_NULL;
    if (!Wp || !aligned(Wp, 256) || Wp_bytes < gbnn_sparse_bytes(C, L, 0)) return GBNN_ERR_WORKSPACE;
    const hipError_t e = launch_sparsify(W, C, L, (int)gbnn_w_row_words(C, L), static_cast<char *>(Wp), Wp_bytes,
                                         status, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GBNN_OK : GBNN_ERR_DEVICE;
}

int gbnn_retrieve_sparse(const void *Wp, size_t Wp_bytes, int C, int L, const int32_t *probes, int64_t K,
                         int max_iters, uint32_t *bits_out, int32_t *symbols_out, int32_t *iters_out, void *stream)
{
    if (!shape_ok(C, L) || L % 32 != 0 || K < 0 || K > GBNN_MAX_K) return GBNN_ERR_SHAPE;
    if (max_iters < 1) return GBNN_ERR_ITERS;
    if (K > 0 && !probes) return GBNN_ERR_NULL;
    if (!Wp || !aligned(Wp, 256) || Wp_bytes < gbnn_sparse_bytes(C, L, 0)) return GBNN_ERR_WORKSPACE;
    const hipError_t e = launch_retrieve_sparse(static_cast<const char *>(Wp), Wp_bytes, C, L,
                                                (int)gbnn_w_row_words(C, L), probes, K, max_iters, bits_out,
                                                symbols_out, iters_out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GBNN_OK : GBNN_ERR_DEVICE;
}

int gbnn_set_kernel_choice(int retrieve_family, int store_kernel)
{
    if (retrieve_family < GBNN_FAMILY_AUTO || retrieve_family > GBNN_FAMILY_WAVE) return GBNN_ERR_RULE;
    if (store_kernel < GBNN_STORE_AUTO || store_kernel > GBNN_STORE_ROWS) return GBNN_ERR_RULE;
    g_retrieve_family.store(retrieve_family, std::memory_order_relaxed);
    g_store_kernel.store(store_kernel, std::memory_order_relaxed);
    return GBNN_OK;
}

const char *gbnn_strerror(int code)
{
    switch (code) {
    case GBNN_OK: return "ok";
    case GBNN_ERR_NULL: return "a required pointer is NULL";
    case GBNN_ERR_SHAPE: return "shape outside the limits (2 <= C <= 64, L >= 1, C*L <= 16384, 0 <= K < 2^31, M >= 0)";
    case GBNN_ERR_RULE: return "unknown retrieval rule";
    case GBNN_ERR_GAMMA: return "gamma outside [0, 32767]";
    case GBNN_ERR_ITERS: return "max_iters must be at least 1";
    case GBNN_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned, or smaller than gbnn_workspace_bytes";
    case GBNN_ERR_DEVICE: return "the HIP runtime refused a kernel launch";
    case GBNN_ERR_TOO_LARGE: return "gbnn_retrieve_static serves networks of up to 8192 neurons (clusters padded to a power of two)";
    default: return "unknown status code";
    }
}

const char *gbnn_retrieve_path(int C, int L, int rule, const void *V0, const void *V_out)
{
    if (!shape_ok(C, L) || !rule_ok(rule)) return nullptr;
    switch (pick_path(C, L, rule, V0, V_out)) {
    case 1: return "wave1";
    case 2: return "wave2";
    case 4: return "wave4";
    case 8: return "wave8";
    case kHalfPath: return "half1";
    default: return "generic";
    }
}

int gbnn_reference_copy(void *dst, const void *src, size_t bytes, int streaming, void *stream)
{
    if (bytes == 0) return GBNN_OK;
    if (!dst || !src) return GBNN_ERR_NULL;
    if (bytes % 16 != 0 || !aligned(dst, 16) || !aligned(src, 16)) return GBNN_ERR_SHAPE;
    const size_t blocks = (bytes + 8191) / 8192;
    if (blocks > 0x7FFFFFFFull) return GBNN_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (streaming)
        hipLaunchKernelGGL(gbnn::k_reference_copy<true>, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const uint8_t *>(src),
                           static_cast<uint8_t *>(dst), bytes);
    else
        hipLaunchKernelGGL(gbnn::k_reference_copy<false>, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const uint8_t *>(src),
                           static_cast<uint8_t *>(dst), bytes);
    return hipGetLastError() == hipSuccess ? GBNN_OK : GBNN_ERR_DEVICE;
}

}  // extern "C"
