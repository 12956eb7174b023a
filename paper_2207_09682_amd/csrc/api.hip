// C-ABI entry points of libqgbdt: argument checks, context and workspace
// management, and the stand-alone forms of the steps (the kernels themselves live
// next to their launchers).
#include <algorithm>
#include <stdarg.h>
#include <string.h>

#include <new>

#include "split_device.h"

static char g_create_error[512] = "";

// Fixed scratch for the entry point that allocates nothing (qgbdt_find_best_splits_static): every GPU the
// library runs on holds its own copy of this array until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; the address kernels are given is looked up once per device (in
// qgbdt_create, with that device current) and kept here.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)4 << 20;
constexpr int STATIC_SCRATCH_DEVICES = 64;
static __device__ __align__(256) unsigned char g_static_scratch[STATIC_SCRATCH_BYTES];
static void* g_static_scratch_ptr[STATIC_SCRATCH_DEVICES] = {};

namespace qgbdt {

int set_error(qgbdt_ctx* ctx, int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx ? ctx->err : g_create_error, 512, fmt, ap);
    va_end(ap);
    return code;
}

// sums of g~, h~ and |g~| over a row set (totals[0..2]): for the overflow check when the a-priori bound cannot rule
// overflow out, and for completing a stand-alone histogram whose most frequent bins were left out
__global__ __launch_bounds__(256) void gh_totals_kernel(const int16_t* __restrict__ gh, const int32_t* __restrict__ idx,
                                                        int64_t begin, int64_t count, int64_t* totals) {
    int64_t sh = 0, sa = 0, sg = 0;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, nthr = (int64_t)gridDim.x * blockDim.x;
    int64_t done = 0;
    if (!idx) {
        // contiguous rows: eight packed values per 16-byte load once the address is aligned
        const int16_t* base = gh + begin;
        int64_t head = (int64_t)(((16 - ((uintptr_t)base & 15)) & 15) >> 1);
        if (head > count) head = count;
        const int64_t n8 = (count - head) >> 3;
        for (int64_t j = tid; j < n8; j += nthr) {
            const uint4 q = *reinterpret_cast<const uint4*>(base + head + 8 * j);
            const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int lo = (int)(int16_t)(w[k] & 0xffffu), hi = (int)(int16_t)(w[k] >> 16);
                sh += (lo & 0xff) + (hi & 0xff);
                sa += abs(lo >> 8) + abs(hi >> 8);
                sg += (lo >> 8) + (hi >> 8);
            }
        }
        // the unaligned head and the tail of fewer than eight values
        for (int64_t p = tid; p < head; p += nthr) { const int v = base[p]; sh += v & 0xff; sa += abs(v >> 8); sg += v >> 8; }
        for (int64_t p = head + 8 * n8 + tid; p < count; p += nthr) { const int v = base[p]; sh += v & 0xff; sa += abs(v >> 8); sg += v >> 8; }
        done = count;
    }
    for (int64_t p = done + tid; p < count; p += nthr) {
        const int64_t i = (int64_t)idx[begin + p];
        const int v = gh[i];
        sh += v & 0xff;
        sa += abs(v >> 8);
        sg += v >> 8;
    }
    for (int o = 32; o > 0; o >>= 1) { sh += __shfl_xor(sh, o); sa += __shfl_xor(sa, o); sg += __shfl_xor(sg, o); }
    // one set of atomics per workgroup: atomics on one address serialize at the memory side (~20 ns each)
    __shared__ int64_t part[3][4];
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { part[0][wave] = sg; part[1][wave] = sh; part[2][wave] = sa; }
    __syncthreads();
    if (threadIdx.x < 3) {
        const int64_t v = part[threadIdx.x][0] + part[threadIdx.x][1] + part[threadIdx.x][2] + part[threadIdx.x][3];
        if (v != 0) atomicAdd((unsigned long long*)&totals[threadIdx.x], (unsigned long long)v);
    }
}
__global__ void zero3_kernel(int64_t* t) {
    if (threadIdx.x < 3) t[threadIdx.x] = 0;
}
__global__ void fill_bytes_kernel(unsigned char* p, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

// Sizes that follow from the shape alone.
static void derive_sizes(qgbdt_ctx* c) {
    const int L = c->shape.max_leaves;
    c->batch_max = L;
    c->max_expand = 3 * L;
    c->max_nodes = 2 * c->max_expand + 1;
    c->max_seg = (int)(c->shape.n_rows / PART_SEG) + c->batch_max + 2;
}

// Bytes of the row groups' slots (local bins handed over to the reduce kernel): the largest any plan of this
// shape asks for -- either word width, with or without the large tiles of frequent-bin skipping; the tile
// shape does not depend on the bit widths.
static size_t partial_slot_bytes(const qgbdt_shape& shape) {
    size_t need = 0;
    for (int w = 16; w <= 32; w += 16)
        for (int skew = 0; skew < 2; ++skew) {
            const HistPlan hp = make_hist_plan(shape, 2, 2, w, skew != 0);
            const size_t b = (size_t)hp.max_items * hp.n_tiles * hp.slot_bytes;
            if (b > need) need = b;
        }
    return need;
}

// Walks the sections of the workspace in a fixed order, every section aligned to 256 bytes.  With a base
// address it assigns the context's pointers, without one it only measures.  Returns the bytes needed.
namespace {
struct Carver {
    unsigned char* base;
    size_t off;
    template <typename T>
    void take(T** p, size_t n) {
        off = (off + 255) & ~(size_t)255;
        if (base) *p = reinterpret_cast<T*>(base + off);
        off += (n ? n : 1) * sizeof(T);
    }
};
}  // namespace

static bool shape_allows_ordered(const qgbdt_shape& s) {
    return s.bin_bytes == 1 && s.n_features % 4 == 0 && s.n_features >= 16 && s.n_features <= 64;
}

static size_t carve_workspace(qgbdt_ctx* c, void* base, uint32_t flags) {
    Carver k{static_cast<unsigned char*>(base), 0};
    const qgbdt_shape& sh = c->shape;
    const size_t N = (size_t)sh.n_rows, F = (size_t)sh.n_features;
    const size_t W = F * (size_t)sh.n_bins;
    const size_t L = (size_t)sh.max_leaves;
    for (int b = 0; b < 3; ++b) k.take(&c->idx[b], N);
    for (int b = 0; b < 3; ++b) k.take(&c->ogh[b], N);
    k.take(&c->gh, N);
    k.take(&c->ghf, N);
    k.take(&c->hist_pool, W * (size_t)(c->max_expand + 1));
    {
        unsigned char* pp = nullptr;
        const size_t need = partial_slot_bytes(sh);
        k.take(&pp, need);
        if (base) { c->hist_partials = pp; c->hist_partials_bytes = need; }
    }
    k.take(&c->flags, N);
    k.take(&c->part_counts, (size_t)PART_GROUPS);
    k.take(&c->seg_counts, (size_t)c->max_seg);
    k.take(&c->seg_prefix, (size_t)c->max_seg + 1);
    k.take(&c->absmax_part, (size_t)2 * QUANT_PARTS);
    k.take(&c->qtotals_part, (size_t)3 * QUANT_PARTS);
    k.take(&c->qtotals, 4);
    k.take(&c->delta, 2);
    k.take(&c->nodes, (size_t)c->max_nodes);
    k.take(&c->sorted_idx, (size_t)c->max_nodes);
    k.take(&c->step, 1);
    k.take(&c->batch, (size_t)c->batch_max);
    k.take(&c->cand, (size_t)2 * c->batch_max * F);
    k.take(&c->hist_entries, (size_t)c->batch_max);
    k.take(&c->hist_counts, 2);
    k.take(&c->pwork, 1);
    k.take(&c->scan_items, (size_t)2 * c->batch_max);
    k.take(&c->leaf_node, L);
    k.take(&c->refit_partial, L * REFIT_PARTS * 2);
    k.take(&c->tmp_i64, 8);
    // optional sections
    if (flags & QGBDT_WS_BIND) {
        k.take(&c->bins_t, N * F * (size_t)sh.bin_bytes);
        k.take(&c->mfb, F);
    } else if (base) { c->bins_t = nullptr; c->mfb = nullptr; }
    if ((flags & QGBDT_WS_ROW_COPIES) && shape_allows_ordered(sh)) {
        for (int b = 0; b < 3; ++b) k.take(&c->obins[b], N * F);
    } else if (base) { c->obins[0] = c->obins[1] = c->obins[2] = nullptr; }
    if (flags & QGBDT_WS_BOOST) {
        k.take(&c->gbuf, N);
        k.take(&c->hbuf, N);
    } else if (base) { c->gbuf = nullptr; c->hbuf = nullptr; }
    return (k.off + 255) & ~(size_t)255;
}

static void free_host(qgbdt_ctx* c) {
    if (c->host_state) (void)hipHostFree(c->host_state);
    if (c->ev) {
        for (int i = 0; i < c->ev_cap; ++i)
            if (c->ev[i]) (void)hipEventDestroy(c->ev[i]);
        delete[] c->ev;
        delete[] c->ev_root;
    }
}

int require_workspace(qgbdt_ctx* ctx) {
    if (!ctx->ws_base)
        return set_error(ctx, QGBDT_E_WORKSPACE, "no workspace: call qgbdt_set_workspace first (qgbdt_workspace_bytes gives its size)");
    return QGBDT_OK;
}

}  // namespace qgbdt

namespace qgbdt {

static int check_bits(qgbdt_ctx* ctx, int bits_g, int bits_h) {
    if (bits_g < 2 || bits_g > 8 || !(bits_h == 0 || (bits_h >= 2 && bits_h <= 8)))
        return set_error(ctx, QGBDT_E_INVALID_ARG, "bits_g=%d, bits_h=%d outside 2..8 (bits_h = 0: constant hessians)", bits_g, bits_h);
    return QGBDT_OK;
}

}  // namespace qgbdt

using namespace qgbdt;

namespace qgbdt {

// Plain streaming read: U 16-byte loads per thread in flight per step, grid-stride; the loaded values are folded
// into a word that is stored only if it takes one particular value, which keeps the loads alive.  NT: loads
// marked non-temporal.
template <int U, bool NT>
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ p, int64_t n16, uint32_t* sink) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    uint32_t acc = 0u;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (NT) {
                const uint32_t* q = reinterpret_cast<const uint32_t*>(p + i + u * stride);
                typedef uint32_t v4 __attribute__((ext_vector_type(4)));
                const v4 t = __builtin_nontemporal_load(reinterpret_cast<const v4*>(q));
                v[u] = make_uint4(t.x, t.y, t.z, t.w);
            } else {
                v[u] = p[i + u * stride];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = p[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u) *sink = acc;
}

}  // namespace qgbdt

extern "C" {

static int check_shape(const qgbdt_shape* shape) {
    if (!shape) return set_error(nullptr, QGBDT_E_INVALID_ARG, "null argument");
    if (shape->bin_bytes != 1 && shape->bin_bytes != 2)
        return set_error(nullptr, QGBDT_E_UNSUPPORTED, "bin_bytes=%d: bins are uint8 (1) or uint16 (2)", shape->bin_bytes);
    if (shape->n_rows < 1 || shape->n_rows > 2147483647LL || shape->n_features < 1 || shape->n_bins < 2 ||
        shape->n_bins > (shape->bin_bytes == 2 ? 1024 : 256) || shape->max_leaves < 1)
        return set_error(nullptr, QGBDT_E_INVALID_ARG, "shape out of range (rows %lld, features %d, bins %d, leaves %d)",
                         (long long)shape->n_rows, shape->n_features, shape->n_bins, shape->max_leaves);
    if (shape->max_leaves > TABLE_MAX)
        return set_error(nullptr, QGBDT_E_UNSUPPORTED, "max_leaves=%d: at most %d (the kernels keep a round's table in LDS)",
                         shape->max_leaves, TABLE_MAX);
    // the plan kernel keeps its sort and replay state of all nodes in LDS
    const size_t L = (size_t)shape->max_leaves, max_nodes = 6 * L + 1, p_max = max_nodes + (max_nodes & 1);
    const size_t plan_lds = p_max * 24 + L * 16 + max_nodes * 12 + (4 * L + 8) * 4;
    if (plan_lds + 512 > 160 * 1024)  // (the kernel's few static words come on top)
        return set_error(nullptr, QGBDT_E_UNSUPPORTED, "max_leaves=%d: the growth bookkeeping would need %zu bytes of LDS (limit 160 KB: at most 658 leaves)",
                         shape->max_leaves, plan_lds);
    return QGBDT_OK;
}

int qgbdt_create(qgbdt_ctx** out, const qgbdt_shape* shape, void* stream) {
    if (!out || !shape) return set_error(nullptr, QGBDT_E_INVALID_ARG, "null argument");
    *out = nullptr;
    int rc = check_shape(shape);
    if (rc != QGBDT_OK) return rc;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1)
        return set_error(nullptr, QGBDT_E_HIP, "no HIP device: this library has no CPU path");
    qgbdt_ctx* c = new (std::nothrow) qgbdt_ctx();
    if (!c) return set_error(nullptr, QGBDT_E_ALLOC, "out of host memory");
    memset(c, 0, sizeof(*c));
    c->shape = *shape;
    c->stream = (hipStream_t)stream;
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return set_error(nullptr, QGBDT_E_HIP, "hipGetDevice failed"); }
    derive_sizes(c);
    c->rounds_hint = 10;
    if (c->device >= 0 && c->device < STATIC_SCRATCH_DEVICES) {
        if (!g_static_scratch_ptr[c->device]) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess || !p) {
                delete c;
                return set_error(nullptr, QGBDT_E_HIP, "hipGetSymbolAddress of the fixed scratch array failed");
            }
            g_static_scratch_ptr[c->device] = p;
        }
        c->static_scratch = g_static_scratch_ptr[c->device];
    }
    if (hipHostMalloc(reinterpret_cast<void**>(&c->host_state), sizeof(StepState), hipHostMallocDefault) != hipSuccess)
        rc = set_error(c, QGBDT_E_ALLOC, "hipHostMalloc failed");
    // kernels whose local bins or bookkeeping exceed the default limit of dynamic LDS are told so once
    if (rc == QGBDT_OK) rc = prepare_hist_kernels(c);
    if (rc == QGBDT_OK) rc = prepare_tree_kernels(c);
    if (rc != QGBDT_OK) {
        snprintf(g_create_error, sizeof(g_create_error), "%s", c->err);
        free_host(c);
        delete c;
        return rc;
    }
    *out = c;
    return QGBDT_OK;
}

int qgbdt_destroy(qgbdt_ctx* ctx) {
    if (!ctx) return QGBDT_OK;
    (void)hipStreamSynchronize(ctx->stream);
    free_host(ctx);
    delete ctx;
    return QGBDT_OK;
}

int qgbdt_set_stream(qgbdt_ctx* ctx, void* stream) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    ctx->stream = (hipStream_t)stream;
    return QGBDT_OK;
}

const char* qgbdt_last_error(const qgbdt_ctx* ctx) { return ctx ? ctx->err : g_create_error; }

int qgbdt_workspace_bytes(const qgbdt_shape* shape, uint32_t flags, size_t* bytes) {
    if (!bytes) return set_error(nullptr, QGBDT_E_INVALID_ARG, "null argument");
    int rc = check_shape(shape);
    if (rc != QGBDT_OK) return rc;
    if (flags & ~(uint32_t)(QGBDT_WS_BIND | QGBDT_WS_ROW_COPIES | QGBDT_WS_BOOST))
        return set_error(nullptr, QGBDT_E_INVALID_ARG, "unknown workspace flags 0x%x", flags);
    qgbdt_ctx tmp;
    memset(&tmp, 0, sizeof(tmp));
    tmp.shape = *shape;
    derive_sizes(&tmp);
    *bytes = carve_workspace(&tmp, nullptr, flags);
    return QGBDT_OK;
}

int qgbdt_set_workspace(qgbdt_ctx* ctx, void* dev, size_t bytes, uint32_t flags) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (flags & ~(uint32_t)(QGBDT_WS_BIND | QGBDT_WS_ROW_COPIES | QGBDT_WS_BOOST))
        return set_error(ctx, QGBDT_E_INVALID_ARG, "unknown workspace flags 0x%x", flags);
    // what was enqueued may still use the old block
    QG_HIP(ctx, hipStreamSynchronize(ctx->stream));
    ctx->ws_base = nullptr;
    ctx->ws_bytes = 0;
    ctx->ws_flags = 0;
    ctx->bound_bins = nullptr;
    ctx->mfb_features = 0;
    if (!dev) return QGBDT_OK;  // detached: every step refuses until a block is set again
    if (((uintptr_t)dev & 255) != 0) return set_error(ctx, QGBDT_E_INVALID_ARG, "the workspace must be 256-byte aligned");
    size_t need = 0;
    {
        qgbdt_ctx tmp = *ctx;
        need = carve_workspace(&tmp, nullptr, flags);
    }
    if (bytes < need)
        return set_error(ctx, QGBDT_E_WORKSPACE, "workspace of %zu bytes is too small: this shape with flags 0x%x needs %zu",
                         bytes, flags, need);
    carve_workspace(ctx, dev, flags);
    ctx->ws_base = dev;
    ctx->ws_bytes = need;
    ctx->ws_flags = flags;
    ctx->ordered = ctx->obins[0] ? 1 : 0;
    hipLaunchKernelGGL(fill_bytes_kernel, dim3(1), dim3(256), 0, ctx->stream, reinterpret_cast<unsigned char*>(ctx->step),
                       (int)sizeof(StepState));
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

int qgbdt_quantize_gradients(qgbdt_ctx* ctx, const float* g, const float* h, int64_t n, int32_t bits_g,
                             int32_t bits_h, uint64_t seed, uint32_t iteration, int32_t rounding, int16_t* gh_out,
                             float* delta_out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!g || !h || !gh_out || !delta_out) return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (int rcw = require_workspace(ctx)) return rcw;
    if (n < 0 || n > ctx->shape.n_rows) return set_error(ctx, QGBDT_E_INVALID_ARG, "n=%lld outside 0..n_rows", (long long)n);
    if (rounding != QGBDT_ROUND_STOCHASTIC && rounding != QGBDT_ROUND_NEAREST)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "rounding=%d", rounding);
    int rc = check_bits(ctx, bits_g, bits_h);
    if (rc != QGBDT_OK) return rc;
    return launch_quantize(ctx, g, h, n, bits_g, bits_h, seed, iteration, rounding, gh_out, delta_out, nullptr, nullptr);
}

int qgbdt_build_histograms(qgbdt_ctx* ctx, const void* bins, const int16_t* gh, const int32_t* row_idx,
                           int64_t begin, int64_t count, int32_t bits_g, int32_t bits_h, int32_t acc_width,
                           int64_t* hist_out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!bins || !gh || !hist_out) return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (int rcw = require_workspace(ctx)) return rcw;
    if (begin < 0 || count < 0 || begin + count > ctx->shape.n_rows)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "slice [%lld, +%lld) outside 0..n_rows", (long long)begin, (long long)count);
    if (acc_width != 0 && acc_width != 16 && acc_width != 32)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "acc_width=%d (0, 16 or 32)", acc_width);
    if (((uintptr_t)bins & 3) != 0) return set_error(ctx, QGBDT_E_INVALID_ARG, "bins must be 4-byte aligned");
    int rc = check_bits(ctx, bits_g, bits_h);
    if (rc != QGBDT_OK) return rc;
    const int64_t W = (int64_t)ctx->shape.n_features * ctx->shape.n_bins;
    if (count > max_rows_for_width(bits_g, bits_h, 32)) {
        // the a-priori bound fails: use the exact totals of these rows (synchronises)
        int64_t tot[3];
        hipLaunchKernelGGL(zero3_kernel, dim3(1), dim3(64), 0, ctx->stream, ctx->tmp_i64);
        hipLaunchKernelGGL(gh_totals_kernel, dim3(512), dim3(256), 0, ctx->stream, gh, row_idx, begin, count,
                           ctx->tmp_i64);
        QG_HIP(ctx, hipMemcpyAsync(tot, ctx->tmp_i64, sizeof(tot), hipMemcpyDeviceToHost, ctx->stream));
        QG_HIP(ctx, hipStreamSynchronize(ctx->stream));
        if (tot[1] > 0xffffffffLL || tot[2] > 0x7fffffffLL)
            return set_error(ctx, QGBDT_E_OVERFLOW_RISK, "sums of %lld rows do not fit 32|32 packed bins", (long long)count);
    }
    rc = launch_fill_zero(ctx, hist_out, W);
    if (rc != QGBDT_OK) return rc;
    if (count == 0) return QGBDT_OK;
    // most frequent bins of the bound matrix are left out by the wide-row kernels and filled in afterwards
    const uint16_t* mfb = (ctx->mfb_features > 0 && ctx->bound_bins == bins) ? ctx->mfb : nullptr;
    const HistPlan plan = make_hist_plan_for(ctx->shape, bits_g, bits_h, acc_width, count, mfb != nullptr,
                                             row_idx == nullptr && ((uintptr_t)bins & 15) == 0);
    if (mfb && plan.wide_v == 0) mfb = nullptr;  // only those kernels skip
    rc = launch_set_hist_table(ctx, plan, begin, count);
    if (rc != QGBDT_OK) return rc;
    RowSource rows;
    rows.gh_pos = 0;  // the caller's packed gradients are in original row order
    IdxSet idx;
    for (int b = 0; b < 4; ++b) { rows.bins[b] = (const uint8_t*)bins; rows.gh[b] = gh; idx.p[b] = const_cast<int32_t*>(row_idx); }
    rc = launch_hist(ctx, plan, rows, idx, row_idx != nullptr, ((uintptr_t)bins & 15) == 0,
                     ctx->hist_entries, ctx->hist_counts, hist_out,
                     (count + hist_target_rows(plan, count, 1) - 1) / hist_target_rows(plan, count, 1),  // the build's row groups
                     ctx->step, mfb);
    if (rc != QGBDT_OK || !mfb) return rc;
    hipLaunchKernelGGL(zero3_kernel, dim3(1), dim3(64), 0, ctx->stream, ctx->tmp_i64);
    hipLaunchKernelGGL(gh_totals_kernel, dim3(512), dim3(256), 0, ctx->stream, gh, row_idx, begin, count, ctx->tmp_i64);
    QG_HIP(ctx, hipGetLastError());
    return launch_fix_frequent_bins(ctx, hist_out, ctx->tmp_i64, mfb);
}

int qgbdt_bind_bins(qgbdt_ctx* ctx, const void* bins) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    ctx->bound_bins = nullptr;
    ctx->mfb_features = 0;
    if (!bins) return QGBDT_OK;
    if (int rcw = require_workspace(ctx)) return rcw;
    if (!ctx->bins_t)
        return set_error(ctx, QGBDT_E_WORKSPACE, "the workspace has no room for the copy of a bound matrix (set it with QGBDT_WS_BIND)");
    int rc = launch_transpose_bins(ctx, bins, ctx->bins_t);
    if (rc != QGBDT_OK) return rc;
    // Most frequent bins (left out by the wide-row histogram kernels); the host learns how many features have one.
    // Only those kernels can use them, so narrow matrices skip the sampling.
    const HistPlan probe = make_hist_plan(ctx->shape, 2, 2, 0, true);
    if (probe.wide_v > 0) {
        rc = launch_frequent_bins(ctx, ctx->bins_t, ctx->mfb);
        if (rc != QGBDT_OK) return rc;
        std::vector<uint16_t> host((size_t)ctx->shape.n_features);
        QG_HIP(ctx, hipMemcpyAsync(host.data(), ctx->mfb, host.size() * sizeof(uint16_t), hipMemcpyDeviceToHost, ctx->stream));
        QG_HIP(ctx, hipStreamSynchronize(ctx->stream));
        int n = 0;
        for (uint16_t v : host) n += (v != 0xffff) ? 1 : 0;
        // worth the extra compare per bin only when many features have such a bin
        ctx->mfb_features = (2 * n >= ctx->shape.n_features) ? n : 0;
    }
    ctx->bound_bins = bins;
    return QGBDT_OK;
}

int qgbdt_subtract_histograms(qgbdt_ctx* ctx, const int64_t* parent, const int64_t* child, int64_t* sibling_out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!parent || !child || !sibling_out) return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (int rcw = require_workspace(ctx)) return rcw;
    return launch_subtract(ctx, parent, child, sibling_out, (int64_t)ctx->shape.n_features * ctx->shape.n_bins);
}

int qgbdt_find_best_splits(qgbdt_ctx* ctx, const int64_t* hist, int32_t n_hists, const qgbdt_leafstat* stats,
                           const float* delta, int32_t min_data_in_leaf, double min_sum_hessian, qgbdt_split* out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!hist || !stats || !delta || !out) return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (int rcw = require_workspace(ctx)) return rcw;
    if (n_hists < 0) return set_error(ctx, QGBDT_E_INVALID_ARG, "n_hists=%d", n_hists);
    return run_find_best_splits(ctx, hist, n_hists, stats, delta, min_data_in_leaf, min_sum_hessian, out,
                                2 * ctx->batch_max, ctx->scan_items, ctx->cand, reinterpret_cast<int32_t*>(ctx->tmp_i64));
}

int qgbdt_find_best_splits_static(qgbdt_ctx* ctx, const int64_t* hist, int32_t n_hists, const qgbdt_leafstat* stats,
                                  const float* delta, int32_t min_data_in_leaf, double min_sum_hessian, qgbdt_split* out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!hist || !stats || !delta || !out) return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (n_hists < 0) return set_error(ctx, QGBDT_E_INVALID_ARG, "n_hists=%d", n_hists);
    if (!ctx->static_scratch) return set_error(ctx, QGBDT_E_UNSUPPORTED, "no fixed scratch on device %d", ctx->device);
    // the array holds: the item count [256 bytes], one item per histogram, one candidate per (histogram, feature)
    const size_t F = (size_t)ctx->shape.n_features;
    const size_t items_off = 256;
    const size_t cand_off = (items_off + (size_t)n_hists * sizeof(ScanItem) + 255) & ~(size_t)255;
    const size_t need = cand_off + (size_t)n_hists * F * sizeof(FeatCand);
    if (need > STATIC_SCRATCH_BYTES)
        return set_error(ctx, QGBDT_E_INVALID_ARG,
                         "n_hists=%d x %d features needs %zu bytes of scratch, the fixed array holds %zu (at most %zu histograms of this shape)",
                         n_hists, ctx->shape.n_features, need, STATIC_SCRATCH_BYTES,
                         (STATIC_SCRATCH_BYTES - 512) / (sizeof(ScanItem) + F * sizeof(FeatCand)));
    if (n_hists == 0) return QGBDT_OK;
    unsigned char* base = static_cast<unsigned char*>(ctx->static_scratch);
    return run_find_best_splits(ctx, hist, n_hists, stats, delta, min_data_in_leaf, min_sum_hessian, out, n_hists,
                                reinterpret_cast<ScanItem*>(base + items_off), reinterpret_cast<FeatCand*>(base + cand_off),
                                reinterpret_cast<int32_t*>(base));
}

int qgbdt_partition_rows(qgbdt_ctx* ctx, const void* bins, int32_t* row_idx, int64_t begin, int64_t count,
                         int32_t feature, int32_t bin, int64_t* n_left_out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!bins || !row_idx || !n_left_out) return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (int rcw = require_workspace(ctx)) return rcw;
    if (begin < 0 || count < 0 || begin + count > ctx->shape.n_rows)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "slice [%lld, +%lld) outside 0..n_rows", (long long)begin, (long long)count);
    if (feature < 0 || feature >= ctx->shape.n_features)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "feature=%d", feature);
    return run_partition_rows(ctx, (const uint8_t*)bins, row_idx, begin, count, feature, bin, n_left_out);
}

int qgbdt_refit_leaves(qgbdt_ctx* ctx, const float* g, const float* h, const int32_t* row_idx,
                       const int64_t* leaf_begin, const int64_t* leaf_count, int32_t n_leaves, double* value_out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!g || !h || !row_idx || !leaf_begin || !leaf_count || !value_out)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (int rcw = require_workspace(ctx)) return rcw;
    if (n_leaves < 0 || n_leaves > ctx->shape.max_leaves)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "n_leaves=%d outside 0..max_leaves", n_leaves);
    return launch_refit(ctx, g, h, nullptr, row_idx, leaf_begin, leaf_count, n_leaves, nullptr, value_out);
}

int qgbdt_grow_tree(qgbdt_ctx* ctx, const void* bins, const float* g, const float* h, const qgbdt_params* p,
                    uint32_t iteration, const qgbdt_tree* t, int32_t* row_idx_out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!bins || !g || !h || !p || !t || !row_idx_out) return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (int rcw = require_workspace(ctx)) return rcw;
    if (!t->n_leaves || !t->split_leaf || !t->split_feature || !t->split_bin || !t->split_gain || !t->split_stats ||
        !t->split_n_left || !t->leaf_begin || !t->leaf_count || !t->leaf_sum_g || !t->leaf_sum_h || !t->leaf_value ||
        !t->leaf_value_quant || !t->delta || !t->hist_units)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer in qgbdt_tree");
    if (p->num_leaves < 1 || p->num_leaves > ctx->shape.max_leaves)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "num_leaves=%d outside 1..max_leaves", p->num_leaves);
    if (p->rounding != QGBDT_ROUND_STOCHASTIC && p->rounding != QGBDT_ROUND_NEAREST)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "rounding=%d", p->rounding);
    if (p->acc_width != 0 && p->acc_width != 16 && p->acc_width != 32)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "acc_width=%d (0, 16 or 32)", p->acc_width);
    if (p->row_layout < QGBDT_ROWS_AUTO || p->row_layout > QGBDT_ROWS_ORDERED)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "row_layout=%d (QGBDT_ROWS_*)", p->row_layout);
    if (p->row_layout == QGBDT_ROWS_ORDERED && !shape_allows_ordered(ctx->shape))
        return set_error(ctx, QGBDT_E_UNSUPPORTED,
                         "ordered rows need uint8 bins and 16..64 features that are a multiple of 4 (n_features=%d, bin_bytes=%d)",
                         ctx->shape.n_features, ctx->shape.bin_bytes);
    if (p->row_layout == QGBDT_ROWS_ORDERED && !ctx->ordered)
        return set_error(ctx, QGBDT_E_WORKSPACE, "the workspace has no room for leaf-ordered copies of the rows (set it with QGBDT_WS_ROW_COPIES)");
    if (((uintptr_t)bins & 3) != 0) return set_error(ctx, QGBDT_E_INVALID_ARG, "bins must be 4-byte aligned");
    int rc = check_bits(ctx, p->bits_g, p->bits_h);
    if (rc != QGBDT_OK) return rc;
    return run_grow_tree(ctx, (const uint8_t*)bins, g, h, p, iteration, t, row_idx_out);
}

int qgbdt_logistic_gradients(qgbdt_ctx* ctx, const float* score, const float* label, int64_t n, float* g_out,
                             float* h_out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!score || !label || !g_out || !h_out) return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (int rcw = require_workspace(ctx)) return rcw;
    if (n < 0 || n > ctx->shape.n_rows) return set_error(ctx, QGBDT_E_INVALID_ARG, "n=%lld outside 0..n_rows", (long long)n);
    return launch_logistic_gradients(ctx, score, label, n, g_out, h_out);
}

int qgbdt_update_scores(qgbdt_ctx* ctx, float* score, const int32_t* row_idx, const int64_t* leaf_begin,
                        const int64_t* leaf_count, const double* leaf_value, int32_t n_leaves, double learning_rate) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!score || !row_idx || !leaf_begin || !leaf_count || !leaf_value)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (int rcw = require_workspace(ctx)) return rcw;
    if (n_leaves < 0 || n_leaves > ctx->shape.max_leaves)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "n_leaves=%d outside 0..max_leaves", n_leaves);
    return launch_update_scores(ctx, score, row_idx, leaf_begin, leaf_count, leaf_value, n_leaves, nullptr, learning_rate);
}

int qgbdt_lambdarank_gradients(qgbdt_ctx* ctx, const float* score, const float* relevance, int64_t n,
                               int32_t group_size, float* g_out, float* h_out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!score || !relevance || !g_out || !h_out) return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (int rcw = require_workspace(ctx)) return rcw;
    if (n < 0 || n > ctx->shape.n_rows) return set_error(ctx, QGBDT_E_INVALID_ARG, "n=%lld outside 0..n_rows", (long long)n);
    if (group_size < 1 || group_size > 1024)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "group_size=%d outside 1..1024", group_size);
    return launch_lambdarank_gradients(ctx, score, relevance, n, group_size, g_out, h_out);
}

// loss: 0 binary cross-entropy, 1 lambdarank with queries of group_size rows
static int boost_iteration(qgbdt_ctx* ctx, int loss, int group_size, const void* bins, const float* label, float* score,
                           const qgbdt_params* p, uint32_t iteration, double learning_rate, const qgbdt_tree* t,
                           int32_t* row_idx_out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!label || !score) return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (loss == 1 && (group_size < 1 || group_size > 1024))
        return set_error(ctx, QGBDT_E_INVALID_ARG, "group_size=%d outside 1..1024", group_size);
    const int64_t N = ctx->shape.n_rows;
    if (int rcw = require_workspace(ctx)) return rcw;
    if (!ctx->gbuf || !ctx->hbuf)
        return set_error(ctx, QGBDT_E_WORKSPACE, "the workspace has no room for the loss derivatives (set it with QGBDT_WS_BOOST)");
    int rc = loss == 0 ? launch_logistic_gradients(ctx, score, label, N, ctx->gbuf, ctx->hbuf)
                       : launch_lambdarank_gradients(ctx, score, label, N, group_size, ctx->gbuf, ctx->hbuf);
    if (rc != QGBDT_OK) return rc;
    rc = qgbdt_grow_tree(ctx, bins, ctx->gbuf, ctx->hbuf, p, iteration, t, row_idx_out);  // validates the rest
    if (rc != QGBDT_OK) return rc;
    return launch_update_scores(ctx, score, row_idx_out, t->leaf_begin, t->leaf_count, t->leaf_value,
                                ctx->shape.max_leaves, t->n_leaves, learning_rate);
}

int qgbdt_boost_iteration(qgbdt_ctx* ctx, const void* bins, const float* label, float* score, const qgbdt_params* p,
                          uint32_t iteration, double learning_rate, const qgbdt_tree* t, int32_t* row_idx_out) {
    return boost_iteration(ctx, 0, 0, bins, label, score, p, iteration, learning_rate, t, row_idx_out);
}

int qgbdt_boost_iteration_lambdarank(qgbdt_ctx* ctx, const void* bins, const float* relevance, int32_t group_size,
                                     float* score, const qgbdt_params* p, uint32_t iteration, double learning_rate,
                                     const qgbdt_tree* t, int32_t* row_idx_out) {
    return boost_iteration(ctx, 1, group_size, bins, relevance, score, p, iteration, learning_rate, t, row_idx_out);
}

int qgbdt_set_profiling(qgbdt_ctx* ctx, int32_t on) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (on && !ctx->ev) {
        // handles only; an event is created when a launch first uses its place (profile_events)
        ctx->ev_cap = 8192;
        ctx->ev = new (std::nothrow) hipEvent_t[ctx->ev_cap];
        if (!ctx->ev) { ctx->ev_cap = 0; return set_error(ctx, QGBDT_E_ALLOC, "out of host memory"); }
        memset(ctx->ev, 0, sizeof(hipEvent_t) * ctx->ev_cap);
        ctx->ev_root = new (std::nothrow) unsigned char[ctx->ev_cap / 2];
        if (!ctx->ev_root) { delete[] ctx->ev; ctx->ev = nullptr; ctx->ev_cap = 0; return set_error(ctx, QGBDT_E_ALLOC, "out of host memory"); }
        memset(ctx->ev_root, 0, ctx->ev_cap / 2);
    }
    ctx->profiling = on ? 1 : 0;
    return QGBDT_OK;
}

int qgbdt_read_profile_roots(qgbdt_ctx* ctx, double* root_ms, int64_t* root_launches) {
    if (!ctx || !root_ms || !root_launches) return QGBDT_E_INVALID_ARG;
    QG_HIP(ctx, hipStreamSynchronize(ctx->stream));
    double ms = 0.0;
    int64_t n = 0;
    for (int i = 0; i + 1 < ctx->ev_used; i += 2) {
        if (!ctx->ev_root[i / 2]) continue;
        float t = 0.0f;
        QG_HIP(ctx, hipEventElapsedTime(&t, ctx->ev[i], ctx->ev[i + 1]));
        ms += t;
        n += 1;
    }
    *root_ms = ms;
    *root_launches = n;
    return QGBDT_OK;
}

int qgbdt_read_profile(qgbdt_ctx* ctx, double* hist_ms, int64_t* hist_launches, double* hist_bytes) {
    if (!ctx || !hist_ms || !hist_launches || !hist_bytes) return QGBDT_E_INVALID_ARG;
    QG_HIP(ctx, hipStreamSynchronize(ctx->stream));
    double ms = 0.0;
    for (int i = 0; i + 1 < ctx->ev_used; i += 2) {
        float t = 0.0f;
        QG_HIP(ctx, hipEventElapsedTime(&t, ctx->ev[i], ctx->ev[i + 1]));
        ms += t;
    }
    StepState st;
    QG_HIP(ctx, hipMemcpy(&st, ctx->step, sizeof(st), hipMemcpyDeviceToHost));
    const double F = ctx->shape.n_features, nb = ctx->shape.n_bins;
    // algorithmic bytes: a bin row and a packed (g~,h~) per row, a row id when gathered, one histogram per build
    *hist_bytes = (double)st.prof_rows_contig * (F + 2.0) + (double)st.prof_rows_idx * (F + 2.0 + 4.0) +
                  (double)st.prof_builds * F * nb * 8.0;
    *hist_ms = ms;
    *hist_launches = st.prof_launches;
    ctx->ev_used = 0;
    st.prof_rows_contig = 0; st.prof_rows_idx = 0; st.prof_launches = 0; st.prof_builds = 0;
    QG_HIP(ctx, hipMemcpy(ctx->step, &st, sizeof(st), hipMemcpyHostToDevice));
    return QGBDT_OK;
}

int qgbdt_measure_stream_read(qgbdt_ctx* ctx, const void* buf, int64_t bytes, int32_t reps, double* gbps_out,
                              int32_t* variant_out) {
    if (!ctx) return QGBDT_E_INVALID_ARG;
    if (!buf || !gbps_out) return set_error(ctx, QGBDT_E_INVALID_ARG, "null pointer");
    if (int rcw = require_workspace(ctx)) return rcw;
    if (((uintptr_t)buf & 15) != 0 || bytes < 16 || (bytes & 15) != 0 || reps < 1)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "buf must be 16-byte aligned, bytes a positive multiple of 16, reps >= 1");
    const int64_t n16 = bytes / 16;
    hipEvent_t e0, e1;
    QG_HIP(ctx, hipEventCreate(&e0));
    QG_HIP(ctx, hipEventCreate(&e1));
    uint32_t* sink = reinterpret_cast<uint32_t*>(ctx->tmp_i64 + 7);
    double best = 0.0;
    int bu = 0, bg = 0, bn = 0;
    hipError_t e = hipSuccess;
    // loads in flight per thread x workgroups per CU x plain / non-temporal loads; the best rate is the ceiling
    for (int nt = 0; nt < 2 && e == hipSuccess; ++nt)
        for (int u = 4; u <= 16 && e == hipSuccess; u *= 2)
            for (int per_cu = 4; per_cu <= 32 && e == hipSuccess; per_cu *= 2) {
                int64_t blocks = (n16 + (int64_t)u * 256 - 1) / ((int64_t)u * 256);
                if (blocks > 256 * per_cu) blocks = 256 * per_cu;
                if (blocks < 1) blocks = 1;
                const dim3 grid((unsigned)blocks), block(256);
#define QG_SR(U_, NT_) hipLaunchKernelGGL((stream_read_kernel<U_, NT_>), grid, block, 0, ctx->stream, (const uint4*)buf, n16, sink)
#define QG_SR_ANY()                                                                  \
    do {                                                                             \
        if (nt) { if (u == 4) QG_SR(4, true); else if (u == 8) QG_SR(8, true); else QG_SR(16, true); }   \
        else    { if (u == 4) QG_SR(4, false); else if (u == 8) QG_SR(8, false); else QG_SR(16, false); } \
    } while (0)
                QG_SR_ANY();  // untimed
                e = hipEventRecord(e0, ctx->stream);
                for (int r = 0; r < reps && e == hipSuccess; ++r) QG_SR_ANY();
#undef QG_SR_ANY
#undef QG_SR
                if (e == hipSuccess) e = hipEventRecord(e1, ctx->stream);
                if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
                float ms = 0.0f;
                if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
                if (e == hipSuccess) e = hipGetLastError();
                const double gbps = ms > 0.0f ? (double)bytes * reps / ((double)ms * 1e-3) / 1e9 : 0.0;
                if (gbps > best) { best = gbps; bu = u; bg = (int)blocks; bn = nt; }
            }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return set_error(ctx, QGBDT_E_HIP, "stream read measurement failed: %s", hipGetErrorString(e));
    *gbps_out = best;
    if (variant_out) { variant_out[0] = bu; variant_out[1] = bg; variant_out[2] = bn; }
    return QGBDT_OK;
}

int qgbdt_describe_hist_plan(const qgbdt_shape* shape, int32_t bits_g, int32_t bits_h, int32_t acc_width, int32_t skewed,
                             int64_t rows, int32_t n_builds, int64_t* out, int32_t n_out) {
    if (!out || n_out < 25) return set_error(nullptr, QGBDT_E_INVALID_ARG, "out must hold 25 values");
    int rc = check_shape(shape);
    if (rc != QGBDT_OK) return rc;
    if (bits_g < 2 || bits_g > 8 || !(bits_h == 0 || (bits_h >= 2 && bits_h <= 8)) ||
        (acc_width != 0 && acc_width != 16 && acc_width != 32) || rows < 0 || n_builds < 1)
        return set_error(nullptr, QGBDT_E_INVALID_ARG, "bits, acc_width, rows or n_builds out of range");
    // rows > 0 with one build: the plan of a stand-alone build of that many rows (the width may fall back to 64-bit
    // words); else the plan of the batched launches of a tree
    const HistPlan p = (n_builds == 1 && rows > 0) ? make_hist_plan_for(*shape, bits_g, bits_h, acc_width, rows, skewed != 0, true)
                                                   : make_hist_plan(*shape, bits_g, bits_h, acc_width, skewed != 0);
    const int64_t v[25] = {p.ft, p.ftp, p.dpr, p.rows_per_it, p.n_tiles, p.threads, p.lds_bytes, p.chunk_rows,
                           p.max_groups, p.max_lanes, p.min_rows_per_group, p.acc_width, p.hshift, p.flat_lanes,
                           p.flat_rows, p.max_items, p.slot_bytes, p.single_rows, p.pad16, p.wide_v, p.ragged,
                           p.bytewise, hist_target_rows(p, rows, n_builds), (int64_t)partial_slot_bytes(*shape), p.two_level};
    for (int i = 0; i < 25; ++i) out[i] = v[i];
    return QGBDT_OK;
}

int qgbdt_tree_stats(const qgbdt_ctx* ctx, int32_t* out4) {
    if (!ctx || !out4 || !ctx->host_state) return QGBDT_E_INVALID_ARG;
    out4[0] = ctx->host_state->rounds; out4[1] = ctx->host_state->n_expanded;
    out4[2] = ctx->host_state->n_commits; out4[3] = ctx->host_state->n_nodes;
    return QGBDT_OK;
}


}  // extern "C"
