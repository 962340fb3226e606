// Host side of the C ABI declared in include/nfd_attn.h: argument checks, tile schedule,
// kernel selection and launches.  Only nfd_attn_create / nfd_attn_destroy allocate or free;
// no other call allocates, synchronises with the host or issues a memset, so all of them can
// be captured into a HIP graph.
#include "../../include/nfd_attn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "kernels_generic.hpp"
#include "kernels_mfma.hpp"
#include "kernels_mfma16.hpp"
#include "kernels_mfma_bwd.hpp"

struct nfd_attn {
    nfd_dtype_t dtype;
    int device;
    int num_cus;
    void* workspace;
    size_t workspace_bytes;
    size_t plan_limit;  // workspace size the schedule is planned against (== workspace_bytes for created handles)
    char err[256];      // fixed buffer: recording an error never allocates
};

namespace {

constexpr size_t kDefaultWorkspace = (size_t)128 << 20;
// one row of one key split in the workspace: 64 bf16 partial outputs + (max, sum) in fp32
constexpr size_t kPartialRowBytes = nfd::mfma::kD * 2 + 2 * sizeof(float);

// Record an error text in the handle's fixed buffer (printf-style; no allocation) and return the code.
__attribute__((format(printf, 3, 4))) int fail(nfd_attn_t* h, int code, const char* fmt, ...) {
    if (h) {
        va_list ap;
        va_start(ap, fmt);
        std::vsnprintf(h->err, sizeof(h->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

// Launches go to the device that is current on the calling thread; pointers and workspace belong to the
// handle's device.  A mismatch would launch on the wrong device, so it is refused.
int check_device(nfd_attn_t* h) {
    int cur = -1;
    const hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return fail(h, NFD_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (cur != h->device) return fail(h, NFD_ERR_UNSUPPORTED, "the current device is not the handle's device");
    return NFD_OK;
}

int check_hip(nfd_attn_t* h, hipError_t e, const char* what) {
    if (e == hipSuccess) return NFD_OK;
    return fail(h, NFD_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

size_t elem_size(nfd_dtype_t dt) { return dt == NFD_BF16 ? 2 : 4; }

// Largest key bound of a block of query rows [r0, r0 + bm) (Sec. 3.1: a row sees all
// frames up to and including its own).
int64_t kmax_rows(int64_t r_last, int T, int P) { return ((int64_t)P + r_last / T + 1) * T; }

}  // namespace

extern "C" {

int64_t nfd_attn_visible_pairs(int T, int kv_frames, int q_frames) {
    if (T < 1 || q_frames < 1 || kv_frames < q_frames) return -1;
    const int64_t P = (int64_t)kv_frames - q_frames, n = q_frames;
    return (int64_t)T * T * (n * P + n * (n + 1) / 2);
}

int nfd_attn_check_args(nfd_dtype_t dtype, int B, int H, int F, int T, int D, int kv_frames, int q_frames) {
    if (B < 1 || H < 1 || F < 1 || T < 1 || D < 1 || q_frames < 1 || kv_frames < 1) return NFD_ERR_SHAPE;
    if (q_frames > kv_frames) return NFD_ERR_SHAPE;
    if (kv_frames > F) return NFD_ERR_CAPACITY;
    if (dtype != NFD_BF16 && dtype != NFD_FP32) return NFD_ERR_UNSUPPORTED;
    if (D > nfd::kGenericMaxD) return NFD_ERR_UNSUPPORTED;
    // 32-bit row indexing inside the kernels
    if ((int64_t)F * T > (int64_t)1 << 30 || (int64_t)B * H > (int64_t)1 << 24) return NFD_ERR_UNSUPPORTED;
    return NFD_OK;
}

int nfd_attn_plan(nfd_dtype_t dtype, int B, int H, int F, int T, int D, int kv_frames, int q_frames,
                  int num_cus, size_t workspace_limit, nfd_attn_plan_t* plan) {
    if (!plan) return NFD_ERR_NULL;
    const int rc = nfd_attn_check_args(dtype, B, H, F, T, D, kv_frames, q_frames);
    if (rc != NFD_OK) return rc;
    if (num_cus <= 0) num_cus = 256;
    if (workspace_limit == 0) workspace_limit = kDefaultWorkspace;
    const int64_t BH = (int64_t)B * H, Sq = (int64_t)q_frames * T;
    const int P = kv_frames - q_frames;
    nfd_attn_plan_t pl{};
    if (dtype == NFD_BF16 && D == nfd::mfma::kD) {
        pl.kernel = 1;
        pl.block_n = nfd::mfma::kBN;
        int64_t visited = 0, max_tiles = 0;
        // The 32-row blocks of a head are dealt to the query tiles as evenly as they go (see the kernel).
        const int64_t n_blocks = (Sq + 31) / 32;
        auto tile_counts = [&](int block_m) {
            pl.block_m = block_m;
            pl.n_q_tiles = (int)((n_blocks + block_m / 32 - 1) / (block_m / 32));
            visited = 0;
            max_tiles = 0;
            const int lo = (int)(n_blocks / pl.n_q_tiles), hi = (int)(n_blocks % pl.n_q_tiles);
            for (int qt = 0; qt < pl.n_q_tiles; ++qt) {
                int b0, nb;
                nfd::mfma::q_tile_blocks(qt, lo, hi, &b0, &nb);
                const int64_t r_last = std::min<int64_t>(32 * (int64_t)(b0 + nb), Sq) - 1;
                const int64_t nt = (kmax_rows(r_last, T, P) + pl.block_n - 1) / pl.block_n;
                visited += nt;
                max_tiles = std::max(max_tiles, nt);
            }
        };
        // 256-row workgroups (64 rows per wavefront, 2 workgroups per CU) are the throughput shape.  When
        // there are very few query rows (single-frame decode of one sequence), the call's time is the
        // length of a workgroup's chain of key tiles, and 128-row workgroups (32 rows per wavefront, 3 per
        // CU) make the links of it shorter: measured -7 % at one frame of 336 queries x 16 heads, +-2 % at two
        // frames, a loss from four frames on (twice the LDS traffic per FLOP).
        tile_counts(nfd::mfma::kBM);
        int wg_per_cu = 2;
        if (BH * pl.n_q_tiles * 4 < (int64_t)num_cus) {
            tile_counts(nfd::mfma::kBM / 2);
            wg_per_cu = 3;
        }
        // Key splits: only when the query tiles alone cannot fill the chip (cached forms).  The count
        // minimises a small cost model in units of the time one workgroup needs for one key tile when
        // two workgroups share a CU: workgroups run in rounds of 2 per CU; a workgroup that has its CU
        // to itself is about 1.2x faster (measured); every workgroup pays a fixed prologue/epilogue of
        // about three tiles; the combine pass costs a launch plus the write and read of the partials,
        // which grows with rows x splits (about one unit per 30000 row-partials of 136 bytes at HBM speed).
        const int64_t slots = (int64_t)num_cus * wg_per_cu, base = BH * pl.n_q_tiles;
        int splits = 1;
        if (base < slots) {
            const size_t per_split = (size_t)(BH * Sq) * kPartialRowBytes;
            double best = 1e30;
            for (int s = 1; s <= 64 && s <= std::max<int64_t>(1, max_tiles / 2); ++s) {
                if (s > 1 && per_split * s > workspace_limit) break;
                const int64_t wgs = base * s;
                const int64_t rounds = (wgs + slots - 1) / slots;
                const double len = (double)((max_tiles + s - 1) / s) + 3.0;
                const double pace = wgs * 2 <= slots ? 0.83 : 1.0;
                const double combine = s > 1 ? 1.0 + (double)s * (double)(BH * Sq) / 30000.0 : 0.0;
                const double cost = rounds * len * pace + combine;
                if (cost < best) { best = cost; splits = s; }
            }
        }
        pl.n_splits = splits;
        if (BH * pl.n_q_tiles * splits > (int64_t)0x7fffffff) return NFD_ERR_UNSUPPORTED;  // grid size
        pl.n_workgroups = (int)(BH * pl.n_q_tiles * splits);
        pl.key_tiles_visited = visited * BH;
        pl.key_tiles_dense = (int64_t)pl.n_q_tiles * (((int64_t)kv_frames * T + pl.block_n - 1) / pl.block_n) * BH;
        pl.workspace_bytes = splits > 1 ? (size_t)(BH * Sq) * splits * kPartialRowBytes : 0;
    } else {
        pl.kernel = 0;
        pl.block_m = nfd::kGenericWaves;  // one row per wavefront
        pl.block_n = 64;
        pl.n_q_tiles = (int)((Sq + pl.block_m - 1) / pl.block_m);
        pl.n_splits = 1;
        if ((BH * Sq + nfd::kGenericWaves - 1) / nfd::kGenericWaves > (int64_t)0x7fffffff) return NFD_ERR_UNSUPPORTED;
        pl.n_workgroups = (int)((BH * Sq + nfd::kGenericWaves - 1) / nfd::kGenericWaves);
        int64_t visited = 0;
        for (int64_t i = 0; i < Sq; ++i) visited += (kmax_rows(i, T, P) + 63) / 64;
        pl.key_tiles_visited = visited * BH;
        pl.key_tiles_dense = Sq * (((int64_t)kv_frames * T + 63) / 64) * BH;
        pl.workspace_bytes = 0;
    }
    *plan = pl;
    return NFD_OK;
}

int nfd_attn_q_tile_rows(int rows, int n_q_tiles, int q_tile, int* first_row, int* n_rows) {
    if (!first_row || !n_rows) return NFD_ERR_NULL;
    if (rows < 1 || n_q_tiles < 1 || q_tile < 0 || q_tile >= n_q_tiles) return NFD_ERR_SHAPE;
    if (rows > 1 << 30) return NFD_ERR_UNSUPPORTED;  // the row limit of the attention calls (32-bit indexing)
    const int n_blocks = (rows + 31) / 32;
    int b0, nb;
    nfd::mfma::q_tile_blocks(q_tile, n_blocks / n_q_tiles, n_blocks % n_q_tiles, &b0, &nb);
    *first_row = std::min(32 * b0, rows);  // more tiles than blocks (never planned): the surplus tiles are empty
    *n_rows = std::min(32 * (b0 + nb), rows) - *first_row;
    return NFD_OK;
}

int nfd_attn_work_item(int BH, int n_q_tiles, int n_splits, int group_q_tiles, unsigned block, int* bh, int* q_tile,
                       int* split) {
    if (!bh || !q_tile || !split) return NFD_ERR_NULL;
    if (BH < 1 || n_q_tiles < 1 || n_splits < 1) return NFD_ERR_SHAPE;
    const nfd::mfma::WorkItem w = nfd::mfma::work_item_of(block, BH, n_q_tiles, n_splits, group_q_tiles);
    if (!w.valid) return NFD_ERR_SHAPE;
    *bh = w.bh; *q_tile = w.q_tile; *split = w.split;
    return NFD_OK;
}

int nfd_attn_create(nfd_attn_t** out, nfd_dtype_t dtype, int device, size_t workspace_bytes) {
    if (!out) return NFD_ERR_NULL;
    *out = nullptr;
    if (dtype != NFD_BF16 && dtype != NFD_FP32) return NFD_ERR_UNSUPPORTED;
    nfd_attn_t* h = new (std::nothrow) nfd_attn();
    if (!h) return NFD_ERR_ALLOC;
    h->dtype = dtype;
    h->device = device;
    h->workspace = nullptr;
    h->workspace_bytes = workspace_bytes ? workspace_bytes : kDefaultWorkspace;
    h->plan_limit = h->workspace_bytes;
    h->err[0] = 0;
    int prev = 0;
    hipError_t e = hipGetDevice(&prev);
    if (e == hipSuccess) e = hipSetDevice(device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) {
        delete h;
        return NFD_ERR_HIP;
    }
    h->num_cus = prop.multiProcessorCount;
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
        (void)hipSetDevice(prev);
        delete h;
        return NFD_ERR_UNSUPPORTED;  // the kernels are written for CDNA4 only
    }
    e = hipMalloc(&h->workspace, h->workspace_bytes);
    (void)hipSetDevice(prev);
    if (e != hipSuccess) {
        delete h;
        return NFD_ERR_ALLOC;
    }
    *out = h;
    return NFD_OK;
}

int nfd_attn_destroy(nfd_attn_t* h) {
    if (!h) return NFD_OK;
    hipError_t e = hipSuccess;
    if (h->workspace) e = hipFree(h->workspace);
    delete h;
    return e == hipSuccess ? NFD_OK : NFD_ERR_HIP;
}

const char* nfd_last_error(const nfd_attn_t* h) { return h ? h->err : "null handle"; }

static void launch_frame_copy(nfd_attn_t* h, size_t es, void* kd, void* vd, const void* ks, const void* vs, int64_t BH,
                              int64_t head_dst, int64_t head_src, int64_t off_dst, int64_t off_src, int64_t len,
                              hipStream_t st);

// k_scale / v_scale non-null: k and v are the 8-bit caches (see nfd_kvcache_append_fp8).
// k_new / v_new non-null: the query frames' own K/V, to be appended to the caches k, v by this call (they are written).
static int fwd_impl(nfd_attn_t* h, const void* q, const void* k, const void* v, void* out, float* lse, int B,
                    int H, int F, int T, int D, int kv_frames, int q_frames, float scale, void* stream,
                    const float* k_scale = nullptr, const float* v_scale = nullptr, const void* k_new = nullptr,
                    const void* v_new = nullptr) {
    if (!h) return NFD_ERR_NULL;
    if (!q || !k || !v || !out) return fail(h, NFD_ERR_NULL, "q, k, v and out must be non-null");
    const bool kv8 = k_scale != nullptr;
    const bool append = k_new != nullptr;
    nfd_attn_plan_t pl;
    const int rc = nfd_attn_plan(h->dtype, B, H, F, T, D, kv_frames, q_frames, h->num_cus, h->plan_limit, &pl);
    if (rc != NFD_OK) return fail(h, rc, "invalid shape arguments");
    // A schedule that would write partials past the workspace must never reach the device.
    if (pl.workspace_bytes > h->workspace_bytes)
        return fail(h, NFD_ERR_ALLOC, "key-split partials (%zu bytes) exceed the scratch memory (%zu bytes)", pl.workspace_bytes,
                    h->workspace_bytes);
    if (const int dc = check_device(h)) return dc;
    // The matrix-core kernels move 16-byte vectors; a view that starts in the middle of a vector would fault.
    if (pl.kernel == 1 && (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) % 16 != 0 || (uintptr_t)lse % 4 != 0))
        return fail(h, NFD_ERR_UNSUPPORTED, "q, k, v, out must be 16-byte aligned (lse 4-byte)");
    if (kv8 && pl.kernel != 1) return fail(h, NFD_ERR_UNSUPPORTED, "the 8-bit cache is built for bf16 queries and head width 64");
    if (append && pl.kernel == 1 && (((uintptr_t)k_new | (uintptr_t)v_new) % 16 != 0))
        return fail(h, NFD_ERR_UNSUPPORTED, "k_new and v_new must be 16-byte aligned");
    if (!(scale > 0.f)) scale = 1.0f / std::sqrt((float)D);

    nfd::FwdParams p{};
    p.k_scale = k_scale; p.v_scale = v_scale;
    p.Spad = (int)(((int64_t)F * T + 63) / 64 * 64);
    p.q = q; p.k = k; p.v = v; p.out = out;
    p.lse = lse;
    p.BH = B * H;
    p.Sq = q_frames * T;
    p.Sk = kv_frames * T;
    p.Scap = F * T;
    p.T = T;
    p.P = kv_frames - q_frames;
    p.D = D;
    p.n_q_tiles = pl.n_q_tiles;
    {
        const int n_blocks = (p.Sq + 31) / 32;
        p.blocks_lo = n_blocks / pl.n_q_tiles;
        p.n_hi = n_blocks % pl.n_q_tiles;
    }
    p.n_splits = pl.n_splits;
    // K and V of all heads against the 256 MB last-level cache (with room for Q, O and partials)
    p.group_q_tiles = pl.n_splits > 1 && (double)p.BH * p.Sk * nfd::mfma::kD * 2.0 * (kv8 ? 1.0 : 2.0) > 192e6;
    p.scale_log2e = scale * nfd::kLog2e;
    p.Snew0 = 0x7fffffff;
    if (append) {
        // In the matrix-core kernel the workgroups read the new rows where they are and copy them into the cache on
        // the side (at most four 16-byte vectors of each tensor per thread); otherwise a copy launch goes first.
        const int64_t n_vec = (int64_t)p.BH * p.Sq * (nfd::mfma::kD / 8);
        if (pl.kernel == 1 && !kv8 && n_vec <= (int64_t)4 * pl.n_workgroups * nfd::mfma::kWaves * 64) {
            p.k_new = k_new; p.v_new = v_new;
            p.Snew0 = p.P * T;
        } else {
            const int64_t frame_elems = (int64_t)T * D;
            launch_frame_copy(h, elem_size(h->dtype), const_cast<void*>(k), const_cast<void*>(v), k_new, v_new, (int64_t)B * H,
                              (int64_t)F * frame_elems, (int64_t)q_frames * frame_elems, (int64_t)p.P * frame_elems, 0,
                              (int64_t)q_frames * frame_elems, (hipStream_t)stream);
        }
    }
    if (pl.n_splits > 1) {
        p.part_o = (__bf16*)h->workspace;
        p.part_ml = (float*)(p.part_o + (size_t)p.BH * pl.n_splits * p.Sq * nfd::mfma::kD);
    }
    hipStream_t st = (hipStream_t)stream;

    if (pl.kernel == 1) {
        const dim3 grid(pl.n_workgroups), block(nfd::mfma::kWaves * 64);
        if (kv8 && pl.block_m == nfd::mfma::kBM)
            hipLaunchKernelGGL((nfd::mfma::attn_fwd_bf16_d64<2, true>), grid, block, 0, st, p);
        else if (kv8)
            hipLaunchKernelGGL((nfd::mfma::attn_fwd_bf16_d64<1, true>), grid, block, 0, st, p);
        else if (lse && pl.block_m == nfd::mfma::kBM)  // training pair: scores from the queries as given
            hipLaunchKernelGGL((nfd::mfma::attn_fwd_bf16_d64_m16<true>), grid, block, 0, st, p);
        else if (lse)
            hipLaunchKernelGGL((nfd::mfma::attn_fwd_bf16_d64<1, false, true>), grid, block, 0, st, p);
        else if (pl.block_m == nfd::mfma::kBM)
            hipLaunchKernelGGL((nfd::mfma::attn_fwd_bf16_d64_m16<false>), grid, block, 0, st, p);
        else
            hipLaunchKernelGGL((nfd::mfma::attn_fwd_bf16_d64<1, false>), grid, block, 0, st, p);
        if (pl.n_splits > 1) {
            const int64_t total = (int64_t)p.BH * p.Sq * (nfd::mfma::kD / 4);
            hipLaunchKernelGGL(nfd::mfma::attn_combine_d64, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, p);
        }
    } else if (h->dtype == NFD_FP32) {
        hipLaunchKernelGGL(nfd::attn_fwd_generic<float>, dim3(pl.n_workgroups), dim3(nfd::kGenericWaves * 64), 0, st, p);
    } else {
        hipLaunchKernelGGL(nfd::attn_fwd_generic<__bf16>, dim3(pl.n_workgroups), dim3(nfd::kGenericWaves * 64), 0, st, p);
    }
    return check_hip(h, hipGetLastError(), "attention launch");
}

int nfd_block_causal_attn_fwd(nfd_attn_t* h, const void* q, const void* k, const void* v, void* out, int B,
                              int H, int F, int T, int D, int kv_frames, int q_frames, float scale,
                              void* stream) {
    return fwd_impl(h, q, k, v, out, nullptr, B, H, F, T, D, kv_frames, q_frames, scale, stream);
}

// ---- forward for callers that cannot allocate ---------------------------------------------------------
// The key-split partials go to a fixed array in the code object instead of a handle's workspace.  `scratch`
// is only a host-side stand-in for the symbol: the address the kernels get is the one hipGetSymbolAddress
// returns with the device current, looked up once per device and kept in that device's pseudo-handle.
namespace {
constexpr size_t kStaticScratchBytes = NFD_NOALLOC_SCRATCH_BYTES;
constexpr int kStaticMaxDevices = 64;
struct StaticDevice {
    bool ready;
    void* scratch_ptr;  // device address of `scratch` on this device
    int num_cus;
};
StaticDevice g_static_dev[kStaticMaxDevices];
std::mutex g_static_mu;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int nfd_block_causal_attn_fwd_noalloc(nfd_dtype_t dtype, const void* q, const void* k, const void* v, void* out, int B,
                                      int H, int F, int T, int D, int kv_frames, int q_frames, float scale, void* stream,
                                      char* err, size_t err_len) {
    nfd_attn local{};  // pseudo-handle on the stack: nothing is allocated, the error text lands in its buffer
    auto done = [&](int rc) {
        if (err && err_len) {
            std::strncpy(err, rc == NFD_OK ? "" : local.err, err_len - 1);
            err[err_len - 1] = 0;
        }
        return rc;
    };
    if (dtype != NFD_BF16 && dtype != NFD_FP32) return done(fail(&local, NFD_ERR_UNSUPPORTED, "unknown dtype"));
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return done(check_hip(&local, e, "hipGetDevice"));
    if (dev < 0 || dev >= kStaticMaxDevices) return done(fail(&local, NFD_ERR_UNSUPPORTED, "device index beyond the table of this entry point"));
    {
        std::lock_guard<std::mutex> lock(g_static_mu);
        StaticDevice& sd = g_static_dev[dev];
        if (!sd.ready) {  // first call on this device, with it current: where this device keeps its copy of the array
            void* ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !ptr) return done(check_hip(&local, e == hipSuccess ? hipErrorInvalidSymbol : e, "hipGetSymbolAddress(scratch)"));
            hipDeviceProp_t prop;
            e = hipGetDeviceProperties(&prop, dev);
            if (e != hipSuccess) return done(check_hip(&local, e, "hipGetDeviceProperties"));
            if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
                return done(fail(&local, NFD_ERR_UNSUPPORTED, "the kernels are written for gfx950 only"));
            sd.scratch_ptr = ptr;
            sd.num_cus = prop.multiProcessorCount;
            sd.ready = true;
        }
        local.workspace = sd.scratch_ptr;  // never the array's name: that is not a device address
        local.num_cus = sd.num_cus;
    }
    local.dtype = dtype;
    local.device = dev;
    local.workspace_bytes = kStaticScratchBytes;
    // The schedule is the one a handle with the default workspace would get, so the result is bit-identical to
    // nfd_block_causal_attn_fwd's; a call whose partials do not fit the array is refused (NFD_ERR_ALLOC), not re-planned.
    local.plan_limit = kDefaultWorkspace;
    return done(fwd_impl(&local, q, k, v, out, nullptr, B, H, F, T, D, kv_frames, q_frames, scale, stream));
}

int nfd_kvcache_append_attn_fwd(nfd_attn_t* h, const void* q, void* k_cache, void* v_cache, const void* k_new,
                                const void* v_new, void* out, int B, int H, int F, int T, int D, int kv_frames,
                                int q_frames, float scale, void* stream) {
    if (!h) return NFD_ERR_NULL;
    if (!k_new || !v_new) return fail(h, NFD_ERR_NULL, "k_new and v_new must be non-null");
    return fwd_impl(h, q, k_cache, v_cache, out, nullptr, B, H, F, T, D, kv_frames, q_frames, scale, stream, nullptr, nullptr,
                    k_new, v_new);
}

int nfd_block_causal_attn_fwd_lse(nfd_attn_t* h, const void* q, const void* k, const void* v, void* out,
                                  float* lse, int B, int H, int F, int T, int D, int kv_frames, int q_frames,
                                  float scale, void* stream) {
    if (h && !lse) return fail(h, NFD_ERR_NULL, "lse must be non-null");
    return fwd_impl(h, q, k, v, out, lse, B, H, F, T, D, kv_frames, q_frames, scale, stream);
}

int nfd_fp8_cache_bytes(int B, int H, int F, int T, int D, size_t* bytes) {
    if (!bytes) return NFD_ERR_NULL;
    if (B < 1 || H < 1 || F < 1 || T < 1 || D < 1) return NFD_ERR_SHAPE;
    if (D != nfd::mfma::kD) return NFD_ERR_UNSUPPORTED;
    if ((int64_t)F * T > (int64_t)1 << 30 || (int64_t)B * H > (int64_t)1 << 24) return NFD_ERR_UNSUPPORTED;
    const int64_t Spad = ((int64_t)F * T + 63) / 64 * 64;
    *bytes = (size_t)B * H * Spad * D;
    return NFD_OK;
}

int nfd_block_causal_attn_fwd_fp8kv(nfd_attn_t* h, const void* q, const void* k8, const void* v8t,
                                    const float* k_scale, const float* v_scale, void* out, int B, int H, int F,
                                    int T, int D, int kv_frames, int q_frames, float scale, void* stream) {
    if (!h) return NFD_ERR_NULL;
    if (!k_scale || !v_scale) return fail(h, NFD_ERR_NULL, "k_scale and v_scale must be non-null");
    if ((uintptr_t)k_scale % 4 != 0 || (uintptr_t)v_scale % 4 != 0)
        return fail(h, NFD_ERR_UNSUPPORTED, "scales must be 4-byte aligned");
    return fwd_impl(h, q, k8, v8t, out, nullptr, B, H, F, T, D, kv_frames, q_frames, scale, stream, k_scale, v_scale);
}

int nfd_kvcache_append_fp8(nfd_attn_t* h, void* k8, void* v8t, const float* k_scale, const float* v_scale,
                           const void* k_new, const void* v_new, int B, int H, int F, int T, int D, int frame_pos,
                           int n_frames, void* stream) {
    if (!h) return NFD_ERR_NULL;
    if (!k8 || !v8t || !k_scale || !v_scale || !k_new || !v_new)
        return fail(h, NFD_ERR_NULL, "caches, scales and new tensors must be non-null");
    if (B < 1 || H < 1 || F < 1 || T < 1 || D < 1 || n_frames < 0 || frame_pos < 0)
        return fail(h, NFD_ERR_SHAPE, "invalid shape arguments");
    if ((int64_t)frame_pos + n_frames > F) return fail(h, NFD_ERR_CAPACITY, "frame_pos + n_frames exceeds the cache capacity F");
    if (h->dtype != NFD_BF16 || D != nfd::mfma::kD)
        return fail(h, NFD_ERR_UNSUPPORTED, "the 8-bit cache is built for bf16 inputs and head width 64");
    if ((int64_t)F * T > (int64_t)1 << 30 || (int64_t)B * H > (int64_t)1 << 24)
        return fail(h, NFD_ERR_UNSUPPORTED, "shape beyond the 32-bit row indexing of the kernels");
    if (((uintptr_t)k8 | (uintptr_t)v8t | (uintptr_t)k_new | (uintptr_t)v_new) % 16 != 0 ||
        ((uintptr_t)k_scale | (uintptr_t)v_scale) % 4 != 0)
        return fail(h, NFD_ERR_UNSUPPORTED, "caches and new tensors must be 16-byte aligned (scales 4-byte)");
    if (n_frames == 0) return NFD_OK;
    if (const int dc = check_device(h)) return dc;
    const int n_rows = n_frames * T, j0 = frame_pos * T, BH = B * H;
    const int64_t Spad = ((int64_t)F * T + 63) / 64 * 64;
    hipStream_t st = (hipStream_t)stream;
    const unsigned gy = (unsigned)std::min(BH, 65535);
    const unsigned k_blocks = (unsigned)(((int64_t)n_rows * 8 + 255) / 256), v_blocks = (unsigned)((n_rows + 63) / 64);
    hipLaunchKernelGGL(nfd::kvcache_append_fp8, dim3(k_blocks + v_blocks, gy), dim3(256), 0, st, (const __bf16*)k_new,
                       (const __bf16*)v_new, (unsigned char*)k8, (unsigned char*)v8t, k_scale, v_scale, n_rows, Spad, j0,
                       BH, k_blocks);
    return check_hip(h, hipGetLastError(), "8-bit kvcache append launch");
}

int nfd_block_causal_attn_bwd(nfd_attn_t* h, const void* q, const void* k, const void* v, const void* out,
                              const void* dout, const float* lse, void* dq, void* dk, void* dv, int B, int H,
                              int F, int T, int D, int kv_frames, int q_frames, float scale, void* stream) {
    if (!h) return NFD_ERR_NULL;
    if (!q || !k || !v || !out || !dout || !lse || !dq || !dk || !dv)
        return fail(h, NFD_ERR_NULL, "all tensors of the backward call must be non-null");
    const int rc = nfd_attn_check_args(h->dtype, B, H, F, T, D, kv_frames, q_frames);
    if (rc != NFD_OK) return fail(h, rc, "invalid shape arguments");
    const int64_t BH = (int64_t)B * H, Sq = (int64_t)q_frames * T, Sk = (int64_t)kv_frames * T;
    if (h->dtype != NFD_BF16 || D != nfd::mfma::kD) {
        if (const int dc = check_device(h)) return dc;
        // general path: fp32 arithmetic, one wavefront per row
        if ((size_t)(BH * Sq) * sizeof(float) > h->workspace_bytes)
            return fail(h, NFD_ERR_ALLOC, "the per-row workspace of the backward exceeds the handle's workspace");
        const int64_t gq = (BH * Sq + nfd::kGenericWaves - 1) / nfd::kGenericWaves;
        const int64_t gk = (BH * Sk + nfd::kGenericWaves - 1) / nfd::kGenericWaves;
        if (gq > (int64_t)0x7fffffff || gk > (int64_t)0x7fffffff)
            return fail(h, NFD_ERR_UNSUPPORTED, "too many rows for one launch of the general backward");
        if (!(scale > 0.f)) scale = 1.0f / std::sqrt((float)D);
        nfd::BwdGenericParams g{};
        g.q = q; g.k = k; g.v = v; g.out = out; g.dout = dout; g.lse = lse;
        g.delta = (float*)h->workspace;
        g.dq = dq; g.dk = dk; g.dv = dv;
        g.BH = (int)BH; g.Sq = (int)Sq; g.Sk = (int)Sk; g.Scap = F * T; g.T = T; g.P = kv_frames - q_frames; g.D = D;
        g.scale = scale;
        g.scale_log2e = scale * nfd::kLog2e;
        hipStream_t gs = (hipStream_t)stream;
        const dim3 blk(nfd::kGenericWaves * 64);
        if (h->dtype == NFD_BF16) {
            hipLaunchKernelGGL(nfd::attn_bwd_dq_generic<__bf16>, dim3((unsigned)gq), blk, 0, gs, g);
            hipLaunchKernelGGL(nfd::attn_bwd_dkdv_generic<__bf16>, dim3((unsigned)gk), blk, 0, gs, g);
        } else {
            hipLaunchKernelGGL(nfd::attn_bwd_dq_generic<float>, dim3((unsigned)gq), blk, 0, gs, g);
            hipLaunchKernelGGL(nfd::attn_bwd_dkdv_generic<float>, dim3((unsigned)gk), blk, 0, gs, g);
        }
        return check_hip(h, hipGetLastError(), "general backward launch");
    }
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out | (uintptr_t)dout | (uintptr_t)dq | (uintptr_t)dk |
         (uintptr_t)dv) % 16 != 0 || (uintptr_t)lse % 4 != 0)
        return fail(h, NFD_ERR_UNSUPPORTED, "tensors must be 16-byte aligned (lse 4-byte)");
    if ((size_t)(BH * Sq) * 2 * sizeof(float) > h->workspace_bytes)
        return fail(h, NFD_ERR_ALLOC, "the per-row workspace of the backward exceeds the handle's workspace");
    if (!(scale > 0.f)) scale = 1.0f / std::sqrt((float)D);

    nfd::mfma::BwdParams p{};
    p.q = q; p.k = k; p.v = v; p.dout = dout; p.out = out; p.lse = lse;
    p.neg_delta = (float*)h->workspace;
    p.lse2 = p.neg_delta + BH * Sq;
    p.dq = dq; p.dk = dk; p.dv = dv;
    p.BH = (int)BH; p.Sq = (int)Sq; p.Sk = (int)Sk; p.Scap = F * T; p.T = T; p.P = kv_frames - q_frames;
    p.n_q_tiles = (int)((Sq + nfd::mfma::kBM - 1) / nfd::mfma::kBM);
    p.n_k_blocks = (int)((Sk + nfd::mfma::kBwdKeysPerWorkgroup - 1) / nfd::mfma::kBwdKeysPerWorkgroup);
    p.scale = scale;
    p.scale_log2e = scale * nfd::kLog2e;
    if (BH * p.n_q_tiles > (int64_t)0x7fffffff || BH * p.n_k_blocks > (int64_t)0x7fffffff)
        return fail(h, NFD_ERR_UNSUPPORTED, "too many workgroups for one launch of the backward");
    if (const int dc = check_device(h)) return dc;
    hipStream_t st = (hipStream_t)stream;
    const unsigned heads8 = (unsigned)BH;  // one workgroup per (head, item)
    // the dq kernel first: it writes the two per-row vectors that the dk/dv kernel reads
    hipLaunchKernelGGL(nfd::mfma::attn_bwd_dq_bf16_d64, dim3(heads8 * p.n_q_tiles), dim3(256), 0, st, p);
    hipLaunchKernelGGL(nfd::mfma::attn_bwd_dkdv_bf16_d64, dim3(heads8 * p.n_k_blocks), dim3(256), 0, st, p);
    return check_hip(h, hipGetLastError(), "backward launch");
}

// Launch one frame-run copy (see kvcache_copy) of two tensors of equal geometry, or of one (vd == nullptr);
// all counts in elements of es bytes.
static void launch_frame_copy(nfd_attn_t* h, size_t es, void* kd, void* vd, const void* ks, const void* vs, int64_t BH,
                              int64_t head_dst, int64_t head_src, int64_t off_dst, int64_t off_src, int64_t len,
                              hipStream_t st) {
    const bool pair = vd != nullptr;
    const bool vec = (head_dst * es) % 16 == 0 && (head_src * es) % 16 == 0 && (off_dst * es) % 16 == 0 &&
                     (off_src * es) % 16 == 0 && (len * es) % 16 == 0 && ((uintptr_t)kd % 16 == 0) &&
                     ((uintptr_t)vd % 16 == 0) && ((uintptr_t)ks % 16 == 0) && ((uintptr_t)vs % 16 == 0);
    const dim3 block(256);
    auto grid_for = [&](int64_t units) {
        const int64_t gy = std::min<int64_t>(BH, 65535);
        const int64_t want_x = std::max<int64_t>(1, ((int64_t)h->num_cus * 32 + gy - 1) / gy);  // enough blocks to fill the chip
        return dim3((unsigned)std::min<int64_t>((units + 255) / 256, want_x), (unsigned)gy);
    };
    auto go = [&](auto tag, int64_t f) {  // f = elements per unit of the copy type
        typedef decltype(tag) E;
        if (pair)
            hipLaunchKernelGGL((nfd::kvcache_copy<E, true>), grid_for(len / f), block, 0, st, (E*)kd, (E*)vd, (const E*)ks,
                               (const E*)vs, head_dst / f, head_src / f, off_dst / f, off_src / f, len / f, BH);
        else
            hipLaunchKernelGGL((nfd::kvcache_copy<E, false>), grid_for(len / f), block, 0, st, (E*)kd, (E*)nullptr,
                               (const E*)ks, (const E*)nullptr, head_dst / f, head_src / f, off_dst / f, off_src / f,
                               len / f, BH);
    };
    if (vec) go(nfd::u32x4{}, (int64_t)(16 / es));
    else if (es == 1) go((unsigned char)0, 1);
    else if (es == 2) go((uint16_t)0, 1);
    else go((uint32_t)0, 1);
}

// Move frames n_drop .. kv_frames-1 of every head to frames 0 .. of the same tensors (two of equal geometry,
// or one when b == nullptr): heads of head elements each, fe elements per frame, es bytes per element.
static void shift_frames(nfd_attn_t* h, size_t es, void* a, void* b, int64_t heads, int64_t head, int64_t fe,
                         int kv_frames, int n_drop, hipStream_t st) {
    const int keep = kv_frames - n_drop;
    const size_t half = ((size_t)(heads * keep * fe) * es + 255) / 256 * 256;  // staging bytes per tensor
    if (keep <= n_drop) {
        // source and destination frames are disjoint: one copy inside the tensors
        launch_frame_copy(h, es, a, b, a, b, heads, head, head, 0, (int64_t)n_drop * fe, keep * fe, st);
    } else if ((b ? 2 : 1) * half <= h->workspace_bytes) {
        // overlapping ranges: through the workspace (out, then back)
        void* as = h->workspace;
        void* bs = b ? (char*)h->workspace + half : nullptr;
        launch_frame_copy(h, es, as, bs, a, b, heads, keep * fe, head, 0, (int64_t)n_drop * fe, keep * fe, st);
        launch_frame_copy(h, es, a, b, as, bs, heads, head, keep * fe, 0, 0, keep * fe, st);
    } else {
        // workspace too small: runs of n_drop frames, oldest first; within a run source and destination are disjoint
        for (int f = n_drop; f < kv_frames; f += n_drop) {
            const int n = std::min(n_drop, kv_frames - f);
            launch_frame_copy(h, es, a, b, a, b, heads, head, head, (int64_t)(f - n_drop) * fe, (int64_t)f * fe,
                              (int64_t)n * fe, st);
        }
    }
}

int nfd_kvcache_append(nfd_attn_t* h, void* k_cache, void* v_cache, const void* k_new, const void* v_new, int B,
                       int H, int F, int T, int D, int frame_pos, int n_frames, void* stream) {
    if (!h) return NFD_ERR_NULL;
    if (!k_cache || !v_cache || !k_new || !v_new) return fail(h, NFD_ERR_NULL, "cache and new tensors must be non-null");
    if (B < 1 || H < 1 || F < 1 || T < 1 || D < 1 || n_frames < 0 || frame_pos < 0)
        return fail(h, NFD_ERR_SHAPE, "invalid shape arguments");
    if ((int64_t)frame_pos + n_frames > F) return fail(h, NFD_ERR_CAPACITY, "frame_pos + n_frames exceeds the cache capacity F");
    if (n_frames == 0) return NFD_OK;
    if (const int dc = check_device(h)) return dc;
    const int64_t frame_elems = (int64_t)T * D;
    launch_frame_copy(h, elem_size(h->dtype), k_cache, v_cache, k_new, v_new, (int64_t)B * H, (int64_t)F * frame_elems,
                      (int64_t)n_frames * frame_elems, (int64_t)frame_pos * frame_elems, 0,
                      (int64_t)n_frames * frame_elems, (hipStream_t)stream);
    return check_hip(h, hipGetLastError(), "kvcache append launch");
}

int nfd_kvcache_shift(nfd_attn_t* h, void* k_cache, void* v_cache, int B, int H, int F, int T, int D,
                      int kv_frames, int n_drop, void* stream) {
    if (!h) return NFD_ERR_NULL;
    if (!k_cache || !v_cache) return fail(h, NFD_ERR_NULL, "caches must be non-null");
    if (B < 1 || H < 1 || F < 1 || T < 1 || D < 1 || kv_frames < 0 || n_drop < 0 || n_drop > kv_frames)
        return fail(h, NFD_ERR_SHAPE, "invalid shape arguments");
    if (kv_frames > F) return fail(h, NFD_ERR_CAPACITY, "kv_frames exceeds the cache capacity F");
    if (n_drop == 0 || kv_frames == n_drop) return NFD_OK;
    if (const int dc = check_device(h)) return dc;
    shift_frames(h, elem_size(h->dtype), k_cache, v_cache, (int64_t)B * H, (int64_t)F * T * D, (int64_t)T * D, kv_frames,
                 n_drop, (hipStream_t)stream);
    return check_hip(h, hipGetLastError(), "kvcache shift launch");
}

int nfd_kvcache_shift_fp8(nfd_attn_t* h, void* k8, void* v8t, int B, int H, int F, int T, int D, int kv_frames,
                          int n_drop, void* stream) {
    if (!h) return NFD_ERR_NULL;
    if (!k8 || !v8t) return fail(h, NFD_ERR_NULL, "caches must be non-null");
    if (B < 1 || H < 1 || F < 1 || T < 1 || D < 1 || kv_frames < 0 || n_drop < 0 || n_drop > kv_frames)
        return fail(h, NFD_ERR_SHAPE, "invalid shape arguments");
    if (kv_frames > F) return fail(h, NFD_ERR_CAPACITY, "kv_frames exceeds the cache capacity F");
    if (D != nfd::mfma::kD) return fail(h, NFD_ERR_UNSUPPORTED, "the 8-bit cache is built for head width 64");
    if ((int64_t)F * T > (int64_t)1 << 30 || (int64_t)B * H > (int64_t)1 << 24)
        return fail(h, NFD_ERR_UNSUPPORTED, "shape beyond the 32-bit row indexing of the kernels");
    if (n_drop == 0 || kv_frames == n_drop) return NFD_OK;
    const int64_t Spad = ((int64_t)F * T + 63) / 64 * 64, BH = (int64_t)B * H;
    const int64_t keep_keys = (int64_t)(kv_frames - n_drop) * T;
    if (T % 16 != 0 && h->workspace_bytes < (size_t)keep_keys)  // checked before anything is launched
        return fail(h, NFD_ERR_ALLOC, "the workspace cannot stage one feature row of the 8-bit V cache");
    if (const int dc = check_device(h)) return dc;
    hipStream_t st = (hipStream_t)stream;
    // K codes: BH heads of Spad rows x 64 bytes, a frame = T rows; V codes: BH * 64 feature rows of Spad bytes,
    // a frame = T bytes of each.  (One tensor at a time: the geometries differ.)
    shift_frames(h, 1, k8, nullptr, BH, Spad * D, (int64_t)T * D, kv_frames, n_drop, st);
    if (T % 16 == 0) {  // whole 16-key groups move: the permuted order inside them is untouched
        shift_frames(h, 1, v8t, nullptr, BH * D, Spad, (int64_t)T, kv_frames, n_drop, st);
    } else {
        // key by key through the workspace (plain order there), as many feature rows at a time as fit
        const int64_t rows = BH * D;
        const int64_t fit = (int64_t)(h->workspace_bytes / (size_t)keep_keys);  // >= 1, checked above
        unsigned char* v = (unsigned char*)v8t;
        unsigned char* ws = (unsigned char*)h->workspace;
        for (int64_t r0 = 0; r0 < rows; r0 += fit) {
            const int64_t nr = std::min(fit, rows - r0);
            const dim3 grid((unsigned)std::min<int64_t>((keep_keys + 255) / 256, 1024), (unsigned)std::min<int64_t>(nr, 65535));
            hipLaunchKernelGGL(nfd::v8t_move_keys, grid, dim3(256), 0, st, ws, v + r0 * Spad, nr, keep_keys, Spad, (int64_t)0,
                               (int64_t)n_drop * T, keep_keys, 0, 1, r0);
            hipLaunchKernelGGL(nfd::v8t_move_keys, grid, dim3(256), 0, st, v + r0 * Spad, ws, nr, Spad, keep_keys, (int64_t)0,
                               (int64_t)0, keep_keys, 1, 0, r0);
        }
    }
    return check_hip(h, hipGetLastError(), "8-bit kvcache shift launch");
}

// ---- speculative sampling bookkeeping (host only) ---------------------------------------------
int nfd_spec_init(nfd_spec_t* s, int capacity, int window, int n_spec, int n_prompt, int total) {
    if (!s) return NFD_ERR_NULL;
    if (capacity < 1 || window < 1 || n_spec < 1 || n_prompt < 1 || total < n_prompt) return NFD_ERR_SHAPE;
    if ((int64_t)window + n_spec > capacity || n_prompt > capacity) return NFD_ERR_CAPACITY;
    s->capacity = capacity; s->window = window; s->n_spec = n_spec; s->total = total;
    s->done = n_prompt; s->cached = n_prompt; s->t_offset = 0;
    return NFD_OK;
}

int nfd_spec_next(nfd_spec_t* s, nfd_spec_step_t* step) {
    if (!s || !step) return NFD_ERR_NULL;
    if (s->done >= s->total) return 0;
    step->n_drop = std::max(0, s->cached - s->window);  // keep at most `window` frames of context
    s->cached -= step->n_drop;
    s->t_offset += step->n_drop;
    step->n_frames = std::min(s->n_spec, s->total - s->done);
    step->frame_pos = s->cached;
    step->kv_frames = s->cached + step->n_frames;
    step->q_frames = step->n_frames;
    step->t_offset = s->t_offset;
    return 1;
}

int nfd_spec_accept(nfd_spec_t* s, const nfd_spec_step_t* step, const int32_t* actions, int action_dim,
                    int* accepted) {
    if (!s || !step || !actions || !accepted) return NFD_ERR_NULL;
    if (action_dim < 1 || step->n_frames < 1 || s->done + step->n_frames > s->total) return NFD_ERR_SHAPE;
    // frames were generated under the action of frame `done` repeated: keep the leading run that matches
    const int32_t* a0 = actions + (int64_t)s->done * action_dim;
    int n = 1;
    for (; n < step->n_frames; ++n) {
        const int32_t* an = actions + (int64_t)(s->done + n) * action_dim;
        bool same = true;
        for (int d = 0; d < action_dim; ++d) same = same && an[d] == a0[d];
        if (!same) break;
    }
    *accepted = n;
    s->done += n;
    s->cached = step->frame_pos + n;  // the rejected frames' K/V are simply overwritten by the next append
    return NFD_OK;
}

int nfd_rope_check_args(nfd_dtype_t dtype, int B, int H, int F, int T, int D, int frame_pos, int n_frames,
                        int grid_h, int grid_w, int n_t, int n_h, int n_w) {
    if (B < 1 || H < 1 || F < 1 || T < 1 || D < 1 || n_frames < 0 || frame_pos < 0) return NFD_ERR_SHAPE;
    if (grid_h < 1 || grid_w < 1 || (int64_t)grid_h * grid_w != T) return NFD_ERR_SHAPE;
    if (n_t < 0 || n_h < 0 || n_w < 0 || ((n_t | n_h | n_w) & 1) || (int64_t)n_t + n_h + n_w != D) return NFD_ERR_SHAPE;
    if ((int64_t)frame_pos + n_frames > F) return NFD_ERR_CAPACITY;
    if (dtype != NFD_BF16 && dtype != NFD_FP32) return NFD_ERR_UNSUPPORTED;
    if (D > 2 * nfd::kRopeMaxPairs) return NFD_ERR_UNSUPPORTED;
    if ((int64_t)F * T > (int64_t)1 << 30 || (int64_t)B * H > (int64_t)1 << 24) return NFD_ERR_UNSUPPORTED;
    return NFD_OK;
}

// k_scale / v_scale non-null: k_cache and v_cache are the 8-bit caches.
static int rope_impl(nfd_attn_t* h, const void* q, void* q_out, void* k_cache, void* v_cache, const void* k_new,
                     const void* v_new, int B, int H, int F, int T, int D, int frame_pos, int n_frames, int t_offset,
                     int grid_h, int grid_w, int n_t, int n_h, int n_w, float theta, void* stream,
                     const float* k_scale, const float* v_scale) {
    if (!h) return NFD_ERR_NULL;
    if (!q || !q_out || !k_cache || !v_cache || !k_new || !v_new) return fail(h, NFD_ERR_NULL, "tensors must be non-null");
    const int rc = nfd_rope_check_args(h->dtype, B, H, F, T, D, frame_pos, n_frames, grid_h, grid_w, n_t, n_h, n_w);
    if (rc != NFD_OK) return fail(h, rc, "invalid rotary-embedding arguments");
    const bool kv8 = k_scale != nullptr;
    if (kv8) {
        if (h->dtype != NFD_BF16 || D != nfd::mfma::kD)
            return fail(h, NFD_ERR_UNSUPPORTED, "the 8-bit cache is built for bf16 inputs and head width 64");
        const uintptr_t any = (uintptr_t)q | (uintptr_t)q_out | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)k_new | (uintptr_t)v_new;
        if (any % 16 != 0 || ((uintptr_t)k_scale | (uintptr_t)v_scale) % 4 != 0)
            return fail(h, NFD_ERR_UNSUPPORTED, "tensors must be 16-byte aligned (scales 4-byte)");
    }
    if (n_frames == 0) return NFD_OK;
    if (const int dc = check_device(h)) return dc;
    const double th = theta > 0.f ? (double)theta : 10000.0;
    nfd::RopeTable tab{};
    {
        const int width[3] = {n_t, n_h, n_w};
        int p = 0;
        for (int ax = 0; ax < 3; ++ax)
            for (int i = 0; i < width[ax] / 2; ++i, ++p) {
                tab.inv_freq[p] = std::pow(th, -2.0 * (double)i / (double)width[ax]);
                tab.axis[p] = (unsigned char)ax;
            }
    }
    nfd::RopeParams rp{};
    rp.BH = B * H; rp.F = F; rp.T = T; rp.D = D;
    rp.frame_pos = frame_pos; rp.n_frames = n_frames;
    rp.t_pos0 = t_offset + frame_pos;
    rp.grid_w = grid_w;
    const size_t es = elem_size(h->dtype);
    {   // a feature pair is the smallest unit a thread loads
        const uintptr_t any = (uintptr_t)q | (uintptr_t)q_out | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)k_new | (uintptr_t)v_new;
        if (any % (2 * es) != 0) return fail(h, NFD_ERR_UNSUPPORTED, "tensors must be aligned to one feature pair");
    }
    const bool aligned = ((uintptr_t)q % 16 == 0) && ((uintptr_t)q_out % 16 == 0) && ((uintptr_t)k_cache % 16 == 0) &&
                         ((uintptr_t)v_cache % 16 == 0) && ((uintptr_t)k_new % 16 == 0) && ((uintptr_t)v_new % 16 == 0);
    const int wide = (int)(16 / es);  // features per 16-byte chunk
    const int vec = (aligned && D % wide == 0) ? wide : 2;
    const int64_t items = (int64_t)n_frames * T * (D / vec);
    const int64_t gx = (items + 255) / 256;
    // enough workgroups to fill the chip, otherwise as many heads per thread as possible (the
    // cosines and sines are shared by all heads)
    const int64_t want_y = std::min<int64_t>(rp.BH, std::max<int64_t>(1, ((int64_t)h->num_cus * 8 + gx - 1) / gx));
    rp.heads_per_thread = (int)((rp.BH + want_y - 1) / want_y);
    const unsigned gy = (unsigned)((rp.BH + rp.heads_per_thread - 1) / rp.heads_per_thread);
    const dim3 grid((unsigned)gx, gy), block(256);
    hipStream_t st = (hipStream_t)stream;
    const nfd::RopeFp8 f8{k_scale, v_scale, ((int64_t)F * T + 63) / 64 * 64};
    if (kv8) {  // vec == 8 here: bf16, D = 64, all tensors 16-byte aligned
        hipLaunchKernelGGL((nfd::rope_kvcache_append<__bf16, 8, true>), grid, block, 0, st, (const __bf16*)q, (__bf16*)q_out,
                           (__bf16*)k_cache, (__bf16*)v_cache, (const __bf16*)k_new, (const __bf16*)v_new, rp, tab, f8);
    } else if (h->dtype == NFD_BF16) {
        if (vec == 8)
            hipLaunchKernelGGL((nfd::rope_kvcache_append<__bf16, 8, false>), grid, block, 0, st, (const __bf16*)q, (__bf16*)q_out,
                               (__bf16*)k_cache, (__bf16*)v_cache, (const __bf16*)k_new, (const __bf16*)v_new, rp, tab, f8);
        else
            hipLaunchKernelGGL((nfd::rope_kvcache_append<__bf16, 2, false>), grid, block, 0, st, (const __bf16*)q, (__bf16*)q_out,
                               (__bf16*)k_cache, (__bf16*)v_cache, (const __bf16*)k_new, (const __bf16*)v_new, rp, tab, f8);
    } else {
        if (vec == 4)
            hipLaunchKernelGGL((nfd::rope_kvcache_append<float, 4, false>), grid, block, 0, st, (const float*)q, (float*)q_out,
                               (float*)k_cache, (float*)v_cache, (const float*)k_new, (const float*)v_new, rp, tab, f8);
        else
            hipLaunchKernelGGL((nfd::rope_kvcache_append<float, 2, false>), grid, block, 0, st, (const float*)q, (float*)q_out,
                               (float*)k_cache, (float*)v_cache, (const float*)k_new, (const float*)v_new, rp, tab, f8);
    }
    return check_hip(h, hipGetLastError(), "rotary embedding launch");
}

int nfd_rope_kvcache_append(nfd_attn_t* h, const void* q, void* q_out, void* k_cache, void* v_cache,
                            const void* k_new, const void* v_new, int B, int H, int F, int T, int D,
                            int frame_pos, int n_frames, int t_offset, int grid_h, int grid_w, int n_t,
                            int n_h, int n_w, float theta, void* stream) {
    return rope_impl(h, q, q_out, k_cache, v_cache, k_new, v_new, B, H, F, T, D, frame_pos, n_frames, t_offset, grid_h,
                     grid_w, n_t, n_h, n_w, theta, stream, nullptr, nullptr);
}

int nfd_rope_kvcache_append_fp8(nfd_attn_t* h, const void* q, void* q_out, void* k8, void* v8t, const float* k_scale,
                                const float* v_scale, const void* k_new, const void* v_new, int B, int H, int F,
                                int T, int D, int frame_pos, int n_frames, int t_offset, int grid_h, int grid_w,
                                int n_t, int n_h, int n_w, float theta, void* stream) {
    if (!h) return NFD_ERR_NULL;
    if (!k_scale || !v_scale) return fail(h, NFD_ERR_NULL, "k_scale and v_scale must be non-null");
    return rope_impl(h, q, q_out, k8, v8t, k_new, v_new, B, H, F, T, D, frame_pos, n_frames, t_offset, grid_h, grid_w,
                     n_t, n_h, n_w, theta, stream, k_scale, v_scale);
}

}  // extern "C"
