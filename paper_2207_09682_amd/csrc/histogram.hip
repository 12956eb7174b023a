// Histogram construction (Algorithm 1 with quantized gradients, Sec. 4.1) with
// workgroup-local packed accumulators in LDS that are combined into the leaf's total
// histogram (hierarchical buffers of Sec. 6.1, packed gradient|hessian words of
// Sec. 6.2, width rule of Sec. 7.4.3).
//
// Bound by HBM traffic on one side -- per row one F-byte bin row, one 2-byte packed
// (g~,h~) and, for a gathered leaf, one 4-byte row id are read once -- and by the
// LDS atomic rate on the other: an LDS atomic costs ~5 clocks per wavefront instruction
// and CU (64-bit ones ~6.5), whatever the number of active lanes and the (<= 4-way) bank
// conflicts, i.e. ~7e12 bin updates/s on the chip, the same order as the ~6e12 bin
// bytes/s that HBM streams.
//
// Work decomposition.  A launch serves a table of histogram builds (one per leaf);
// every build is cut into row groups and the (build, group) pairs are the work
// items the workgroups loop over.  A workgroup accumulates a group chunk by chunk
// (a chunk is as many rows as a 16|16 packed accumulator can take).  The last chunk of
// a group -- the only one when the group fits a chunk, which the group sizing aims
// for -- is handed over as it is: the local bins are copied to the group's slot with plain
// stores and hist_reduce_kernel adds the slots of a build to its histogram.  Earlier
// chunks are merged with 64-bit global atomics (same-address atomics from a thousand
// workgroups serialize at the memory side: four times the cost of the slots).
//
// Local histogram layout: [bin][feature column]; for narrow rows the pitch is 32 words,
// so the LDS bank is the feature; the order in which a lane issues the atomics of
// the four features of a dword is rotated per row so that lanes of one instruction
// spread over the features.  Lanes that have no place in a tile are masked for the
// atomics (they would otherwise hit one word together and serialize).
#include <type_traits>

#include "common.h"

namespace qgbdt {

// Workgroup size of the histogram kernels, and the wavefronts per SIMD their register
// budgets are sized for (second launch-bound: 4 -> at most 128 VGPRs, 8 -> at most 64).
constexpr int HIST_THREADS = 512;
constexpr int HIST_WAVES = 4;

__global__ void fill_zero_kernel(int64_t* p, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0;
}

int launch_fill_zero(qgbdt_ctx* ctx, int64_t* p, int64_t n_words) {
    int blocks = (int)((n_words + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, ctx->stream, p, n_words);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

// Expands the per-row int16 (g~ high byte, h~ low byte) into the packed word that
// is added to a bin: g~ * 2^s + h~, where s is the width of the hessian field: 32 for 64-bit
// words; for 32-bit words 16, or -- when the two bit widths differ -- the split of the 32 bits
// that lets a word take the most rows (Sec. 7.4.3: the field widths follow from the bit widths
// and the number of rows; e.g. 13|19 for 3-bit gradients and 8-bit hessians).
template <int W>
struct Acc;
template <>
struct Acc<16> {
    using word = uint32_t;
    // (g~ << s) + h~ = t * (2^(s-8) - 1) + ghv with t = ghv minus its low byte (one AND, one multiply-add);
    // `mul` = 2^(s-8) - 1
    static __device__ __forceinline__ word expand(int ghv, int mul) { return (word)(__mul24(ghv & ~0xff, mul) + ghv); }
    static __device__ __forceinline__ void add(word* p, word v) { atomicAdd(p, v); }
    static __device__ __forceinline__ int64_t widen(word v, int s) {
        const int64_t G = (int32_t)v >> s;
        const int64_t H = v & ((1u << s) - 1u);
        return G * 4294967296LL + H;
    }
};
template <>
struct Acc<32> {
    using word = unsigned long long;
    static __device__ __forceinline__ word expand(int ghv, int) {
        return (word)((int64_t)(ghv >> 8) * 4294967296LL + (int64_t)(ghv & 0xff));
    }
    static __device__ __forceinline__ void add(word* p, word v) { atomicAdd(p, v); }
    static __device__ __forceinline__ int64_t widen(word v, int) { return (int64_t)v; }
};

// Work item -> (table entry, row group): the builds' first items, ascending, are copied into LDS once per workgroup
// (one load per thread instead of a chain of dependent loads per item) and searched there.
__device__ __forceinline__ void load_item_starts(const HistEntry* __restrict__ entries, int n_entries, int* s_start) {
    for (int t = threadIdx.x; t < n_entries; t += blockDim.x) s_start[t] = entries[t].item_start;
    __syncthreads();
}
__device__ __forceinline__ int find_entry(const int* s_start, int n_entries, int item) {
    int lo = 0, hi = n_entries - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (s_start[mid] <= item) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__device__ __forceinline__ void count_profile(const HistEntry* __restrict__ entries, int n_entries, bool idx,
                                              StepState* step) {
    int64_t rows = 0;
    for (int e = 0; e < n_entries; ++e) rows += entries[e].count;
    if (idx) step->prof_rows_idx += rows; else step->prof_rows_contig += rows;
    step->prof_launches += 1;
    step->prof_builds += n_entries;
}

// Workgroup -> (feature tile, row-group lane) for launches with several feature tiles.  The
// hardware deals consecutive workgroups round-robin to the 8 XCDs (each with its own L2), so
// the T workgroups that read the T tiles of the same rows are made consecutive *within one
// XCD*: they then run at about the same time behind the same L2, every cache line of a row is
// fetched once, and a DRAM page is swept once instead of once per tile.
__device__ __forceinline__ void tile_and_lane(int n_tiles, int& tile, int& glane) {
    const int id = blockIdx.x;
    const int xcd = id & 7, s = id >> 3;
    tile = s % n_tiles;
    glane = (s / n_tiles) * 8 + xcd;
}

// Merge of the local bins into the total histogram and reset of the local bins.
// Both are [bin][feature], so LDS is walked linearly (no bank conflicts) and the
// atomics of a wavefront fall into consecutive words.
// Column of a tile's local bins -> feature of the tile when the layout keeps 4 unused words
// after every 16 features (-1: padding).
__device__ __forceinline__ int unpad16(int col) {
    const int g = col / 20, o = col - 20 * g;
    return o < 16 ? 16 * g + o : -1;
}

template <int W>
__device__ __forceinline__ void merge_local(typename Acc<W>::word* lds, int lds_words, int ftp, int ft, int f0, int F,
                                            int64_t* hist, int hshift, bool pad16 = false) {
    for (int w = threadIdx.x; w < lds_words; w += blockDim.x) {
        const int b = w / ftp;
        int f = w - b * ftp;
        if (pad16) { f = unpad16(f); if (f < 0) continue; }
        const typename Acc<W>::word v = lds[w];
        if (v != 0 && f < ft) {
            lds[w] = 0;
            atomicAdd(reinterpret_cast<unsigned long long*>(hist + (int64_t)b * F + f0 + f),
                      (unsigned long long)Acc<W>::widen(v, hshift));
        }
    }
}

// Last chunk of a row group: the local bins go to the group's slot as they are (plain 16-byte
// stores, padding included) and are reset; the reduce kernel adds the slots of a build to
// its histogram.  Costs a quarter of the same merge through atomics.
template <int W>
__device__ __forceinline__ void store_partial(typename Acc<W>::word* lds, int lds_bytes, unsigned char* slot) {
    uint4* l4 = reinterpret_cast<uint4*>(lds);
    uint4* s4 = reinterpret_cast<uint4*>(slot);
    const int n4 = lds_bytes >> 4;
    for (int i = threadIdx.x; i < n4; i += blockDim.x) {
        s4[i] = l4[i];
        l4[i] = make_uint4(0u, 0u, 0u, 0u);
    }
    const int done = n4 << 4;  // a tile whose bins are not a multiple of 16 bytes
    for (int i = done + 4 * threadIdx.x; i < lds_bytes; i += 4 * blockDim.x) {
        *reinterpret_cast<uint32_t*>(slot + i) = *reinterpret_cast<uint32_t*>(reinterpret_cast<unsigned char*>(lds) + i);
        *reinterpret_cast<uint32_t*>(reinterpret_cast<unsigned char*>(lds) + i) = 0u;
    }
}

// Fast path (feature count a multiple of 4), any row set.  lane -> (row r of the
// iteration, dword q of the row's feature tile); U row-iterations (U*rows_per_it
// <= 64 rows) form one block of a wavefront.  All loads of a block are issued before
// its first LDS atomic and the loads of the wavefront's next block are already in
// flight while the atomics of the current one are issued.  Rows beyond the end and
// lanes without work are not branched around: they read a valid row and add zero.
//
// Instruction budget: the four SIMDs of a CU issue one VALU instruction per clock
// between them and the LDS takes one 64-lane atomic per ~5.7 clocks, so a bin may
// cost ~5 VALU instructions: one bit-field extract and one 24-bit multiply-add
// into the byte address of its LDS word, plus its share of the per-row work.
//
// RAG (feature count not a multiple of 4): rows start at any byte, so the dwords are read
// unaligned, and the last dword of a tile row is moved back to end with the tile row (it then
// overlaps its neighbour and only its upper bytes count), so that no load leaves the row.
// Tiles are at least 4 features wide in this mode.
//
// BB = 2 (16-bit bins, up to 1024 per feature): the same kernel with two bins per dword; "ragged" then means an odd
// feature count (rows start at odd multiples of 2 bytes).
template <bool RAG>
__device__ __forceinline__ uint32_t load_bins4(const uint8_t* p) {
    if (RAG) {
        uint32_t v;
        __builtin_memcpy(&v, p, 4);
        return v;
    }
    return *reinterpret_cast<const uint32_t*>(p);
}

template <int W, bool IDX, int U, bool RAG, int BB>
__global__ __launch_bounds__(HIST_THREADS, HIST_WAVES) void hist_kernel(RowSource src, IdxSet idxs,
                                                    const HistEntry* __restrict__ entries,
                                                    const int32_t* __restrict__ table_counts, int64_t* hist_base,
                                                    unsigned char* partials, int F, int nb, HistPlan plan,
                                                    StepState* step) {
    using word = typename Acc<W>::word;
    constexpr int NPD = 4 / BB;  // bins per dword
    extern __shared__ unsigned char lds_raw[];
    word* lds = reinterpret_cast<word*>(lds_raw);

    const int n_entries = table_counts[0], n_items = table_counts[1];
    const int hmul = (1 << (plan.hshift - 8)) - 1;
    int tile, glane;
    tile_and_lane(plan.n_tiles, tile, glane);
    const int n_lanes = (int)gridDim.x / plan.n_tiles;  // row-group lanes (a multiple of 8)
    if (glane >= n_items) return;
    if (step && blockIdx.x == 0 && threadIdx.x == 0) count_profile(entries, n_entries, IDX, step);

    const int f0 = tile * plan.ft;
    const int ft = min(plan.ft, F - f0);
    const int ftp = plan.ftp;
    const int lds_words = nb * ftp;
    for (int w = threadIdx.x; w < lds_words; w += blockDim.x) lds[w] = 0;
    __shared__ int s_start[TABLE_MAX];
    load_item_starts(entries, n_entries, s_start);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = blockDim.x >> 6;
    const int rpi = plan.rows_per_it;
    int q = lane % plan.dpr, r = lane / plan.dpr;
    const bool lane_on = (r < rpi) && (NPD * q < ft);
    if (!lane_on) { q = 0; r = 0; }
    const int rot = (q >> 3) + r;
    const int nval = RAG ? min(NPD, ft - NPD * q) : NPD;  // features in the lane's dword
    const int back = NPD - nval;                          // bins its load is moved back
    uint32_t sh[NPD], fl4[NPD];  // bit offset of the k-th bin in the dword, byte offset of its feature column in LDS
    bool okk[NPD];
#pragma unroll
    for (int k = 0; k < NPD; ++k) {
        const int c = (k + rot) & (NPD - 1);
        okk[k] = c < nval;
        sh[k] = 8 * BB * (okk[k] ? c + back : 0);
        fl4[k] = (uint32_t)(NPD * q + (okk[k] ? c : 0) + (plan.pad16 ? 4 * (q >> 2) : 0)) * (uint32_t)sizeof(word);
    }
    const uint32_t pitch = (uint32_t)ftp * (uint32_t)sizeof(word);  // LDS bytes per bin row
    const int S = U * rpi;                                          // rows per block of one wavefront
    const int64_t row_bytes = (int64_t)F * BB;

    for (int item = glane; item < n_items; item += n_lanes) {
        const HistEntry en = entries[find_entry(s_start, n_entries, item)];
        const int64_t rows_per_group = (en.count + en.groups - 1) / en.groups;
        const int64_t gbegin = min(en.count, (int64_t)(item - en.item_start) * rows_per_group);
        const int64_t gend = min(en.count, gbegin + rows_per_group);
        int64_t* hist = hist_base + (int64_t)en.slot * F * nb;
        unsigned char* slot = partials + ((size_t)item * plan.n_tiles + tile) * (size_t)plan.slot_bytes;
        const int32_t* idx = IDX ? (idxs.p[en.buf] + en.begin) : nullptr;
        // gathered rows are read from the original arrays, contiguous ones from the entry's buffer
        const int sb = IDX ? BUF_ORIGINAL : en.buf;
        const uint8_t* colbase = src.bins[sb] + (f0 + NPD * q - back) * BB;
        const bool gpos = IDX && src.gh_pos != 0;  // packed gradients in list order
        const int16_t* gh = gpos ? src.gh[en.buf] + en.begin : src.gh[sb];

        // a group without rows still hands over its (empty) bins
        for (int64_t cbegin = gbegin; cbegin < gend || cbegin == gbegin; cbegin += plan.chunk_rows) {
            const int64_t cend = min(gend, cbegin + (int64_t)plan.chunk_rows);
            const int crow = (int)(cend - cbegin);
            __syncthreads();
            const int32_t* ib = IDX ? idx + cbegin : nullptr;
            const int64_t row_base = IDX ? 0 : en.begin + cbegin;
            if (wave * S < crow) {
                // three stages in flight per wavefront: row ids of block n+2, bin dwords and packed
                // gradients of block n+1, LDS atomics of block n
                int64_t rown[U];
                uint32_t d[U], dn[U];
                int gv[U], gn[U];
                {
                    int64_t rows[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int p = min(wave * S + u * rpi + r, crow - 1);
                        rows[u] = IDX ? (int64_t)ib[p] : row_base + p;
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        d[u] = load_bins4<RAG>(colbase + rows[u] * row_bytes);
                        gv[u] = gh[gpos ? cbegin + min(wave * S + u * rpi + r, crow - 1) : rows[u]];
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int p = min((wave + n_waves) * S + u * rpi + r, crow - 1);
                        rown[u] = IDX ? (int64_t)ib[p] : row_base + p;
                    }
                }
                for (int ro = wave * S; ro < crow; ro += n_waves * S) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        dn[u] = load_bins4<RAG>(colbase + rown[u] * row_bytes);
                        gn[u] = gh[gpos ? cbegin + min(ro + n_waves * S + u * rpi + r, crow - 1) : rown[u]];
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {  // row ids two blocks ahead (clamped when past the end)
                        const int p = min(ro + 2 * n_waves * S + u * rpi + r, crow - 1);
                        rown[u] = IDX ? (int64_t)ib[p] : row_base + p;
                    }
                    // lanes without a place in the tile sit out (their loads alias lane 0's: atomics on the
                    // same words would serialize); rows past the end are not branched around, they add zero
                    if (lane_on) {
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const bool ok = ro + u * rpi + r < crow;
                            const word v = Acc<W>::expand(ok ? gv[u] : 0, hmul);
#pragma unroll
                            for (int k = 0; k < NPD; ++k) {
                                const uint32_t b = __builtin_amdgcn_ubfe(d[u], sh[k], 8u * BB);
                                if (!RAG || okk[k])
                                    Acc<W>::add(reinterpret_cast<word*>(lds_raw + (__umul24(b, pitch) + fl4[k])), v);
                            }
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) { d[u] = dn[u]; gv[u] = gn[u]; }
                }
            }
            __syncthreads();
            if (cend >= gend) store_partial<W>(lds, plan.lds_bytes, slot);
            else merge_local<W>(lds, lds_words, ftp, ft, f0, F, hist, plan.hshift, plan.pad16 != 0);
        }
    }
}

// Wide rows (several feature tiles; F and the matrix address multiples of V = 16 or 8 bytes):
// like hist_kernel, but a lane reads V bytes -- lane -> (row r of the iteration, V-byte piece c
// of the tile row) -- so a wavefront instruction brings 1 KB (512 B), several times the bytes in
// flight per register-resident load and a fraction of the address arithmetic per bin.
//  V = 16: local bins keep 4 unused words after every 16 features (pitch 20 words per piece):
//          piece c then starts at bank 20c mod 32, the pieces of a tile row fall on distinct
//          multiples of 4, and with the per-row byte rotation the 64 lanes of every instruction
//          spread over all 32 banks, two lanes each.
//  V = 8:  (tiles of at most 64 features, unpadded) half of the rows swap the two dwords of their
//          piece, which together with the byte rotation spreads an instruction over 32 columns.
template <int W, bool IDX, int V, int U, bool SKIP>
__global__ __launch_bounds__(1024) void hist_wide_kernel(RowSource src, IdxSet idxs,
                                                                    const HistEntry* __restrict__ entries,
                                                                    const int32_t* __restrict__ table_counts,
                                                                    int64_t* hist_base, unsigned char* partials, int F,
                                                                    int nb, HistPlan plan, StepState* step,
                                                                    const uint16_t* __restrict__ mfb) {
    using word = typename Acc<W>::word;
    using vec = typename std::conditional<V == 16, uint4, uint2>::type;
    constexpr int NV = V / 4;  // dwords per lane
    extern __shared__ unsigned char lds_raw[];
    word* lds = reinterpret_cast<word*>(lds_raw);

    const int n_entries = table_counts[0], n_items = table_counts[1];
    const int hmul = (1 << (plan.hshift - 8)) - 1;
    int tile, glane;
    tile_and_lane(plan.n_tiles, tile, glane);
    const int n_lanes = (int)gridDim.x / plan.n_tiles;
    if (glane >= n_items) return;
    if (step && blockIdx.x == 0 && threadIdx.x == 0) count_profile(entries, n_entries, IDX, step);

    const int f0 = tile * plan.ft;
    const int ft = min(plan.ft, F - f0);  // a multiple of V
    const int ftp = plan.ftp;
    const int lds_words = nb * ftp;
    for (int w = threadIdx.x; w < lds_words; w += blockDim.x) lds[w] = 0;
    __shared__ int s_start[TABLE_MAX];
    load_item_starts(entries, n_entries, s_start);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = blockDim.x >> 6;
    const int P = plan.ft / V;  // pieces per tile row (a power of two <= 64)
    const int rpi = 64 / P;     // rows per wavefront instruction
    int c = lane % P;
    const int r = lane / P;
    const bool lane_on = V * c < ft;
    if (!lane_on) c = 0;
    const int rot = r & 3;
    const bool swap = (V == 8) && ((r >> 2) & 1);  // this lane handles its two dwords in the other order
    uint32_t sh[4], flk[4];  // bit offset of the k-th bin in a dword, byte offset of its column for the first dword
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int cc = (k + rot) & 3;
        sh[k] = 8 * cc;
        const int col0 = (V == 16) ? 20 * c : 8 * c + (swap ? 4 : 0);
        flk[k] = (uint32_t)(col0 + cc) * (uint32_t)sizeof(word);
    }
    // Bins that are not accumulated (most frequent bin of a feature, when the caller bound the matrix and the
    // bin holds most of the feature's rows): skip[i][k] is that bin for the column the lane's (i, k)-th atomic
    // goes to, or a value no bin takes.  The split search rebuilds the skipped entry from the leaf's totals.
    uint32_t skipb[SKIP ? NV : 1][4];
    if (SKIP) {
#pragma unroll
        for (int i = 0; i < NV; ++i)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int cc = (k + rot) & 3;
                const int dwi = (V == 16) ? i : (swap ? 1 - i : i);  // which dword of the piece the i-th handled one is
                const int col = f0 + V * c + 4 * dwi + cc;
                skipb[SKIP ? i : 0][k] = (lane_on && col < F) ? (uint32_t)mfb[col] : 0xffffu;
            }
    }
    // byte offset from the first to the second handled dword's columns (V = 8: -4 columns when swapped)
    const uint32_t step2 = (uint32_t)((swap ? -4 : 4) * (int)sizeof(word));
    const uint32_t pitch = (uint32_t)ftp * (uint32_t)sizeof(word);
    const int S = U * rpi;

    for (int item = glane; item < n_items; item += n_lanes) {
        const HistEntry en = entries[find_entry(s_start, n_entries, item)];
        const int64_t rows_per_group = (en.count + en.groups - 1) / en.groups;
        const int64_t gbegin = min(en.count, (int64_t)(item - en.item_start) * rows_per_group);
        const int64_t gend = min(en.count, gbegin + rows_per_group);
        int64_t* hist = hist_base + (int64_t)en.slot * F * nb;
        unsigned char* slot = partials + ((size_t)item * plan.n_tiles + tile) * (size_t)plan.slot_bytes;
        const int32_t* idx = IDX ? (idxs.p[en.buf] + en.begin) : nullptr;
        const int sb = IDX ? BUF_ORIGINAL : en.buf;
        const uint8_t* colbase = src.bins[sb] + f0 + V * c;
        const bool gpos = IDX && src.gh_pos != 0;  // packed gradients in list order
        const int16_t* gh = gpos ? src.gh[en.buf] + en.begin : src.gh[sb];

        for (int64_t cbegin = gbegin; cbegin < gend || cbegin == gbegin; cbegin += plan.chunk_rows) {
            const int64_t cend = min(gend, cbegin + (int64_t)plan.chunk_rows);
            const int crow = (int)(cend - cbegin);
            __syncthreads();
            const int32_t* ib = IDX ? idx + cbegin : nullptr;
            const int64_t row_base = IDX ? 0 : en.begin + cbegin;
            if (wave * S < crow) {
                // three stages in flight: row ids of block n+2, bin pieces and packed gradients of
                // block n+1, LDS atomics of block n; rows past the end re-read the last row and add zero
                int64_t rown[U];
                vec d[U], dn[U];
                int gv[U], gn[U];
                {
                    int64_t rows[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int p = min(wave * S + u * rpi + r, crow - 1);
                        rows[u] = IDX ? (int64_t)ib[p] : row_base + p;
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        d[u] = *reinterpret_cast<const vec*>(colbase + rows[u] * F);
                        gv[u] = gh[gpos ? cbegin + min(wave * S + u * rpi + r, crow - 1) : rows[u]];
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int p = min((wave + n_waves) * S + u * rpi + r, crow - 1);
                        rown[u] = IDX ? (int64_t)ib[p] : row_base + p;
                    }
                }
                for (int ro = wave * S; ro < crow; ro += n_waves * S) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        dn[u] = *reinterpret_cast<const vec*>(colbase + rown[u] * F);
                        gn[u] = gh[gpos ? cbegin + min(ro + n_waves * S + u * rpi + r, crow - 1) : rown[u]];
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int p = min(ro + 2 * n_waves * S + u * rpi + r, crow - 1);
                        rown[u] = IDX ? (int64_t)ib[p] : row_base + p;
                    }
                    if (lane_on) {  // lanes beyond the tile's width sit out (their loads alias piece 0)
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const bool ok = ro + u * rpi + r < crow;
                        const word v = Acc<W>::expand(ok ? gv[u] : 0, hmul);
                        uint32_t dw[4];
                        if constexpr (V == 16) {
                            dw[0] = d[u].x; dw[1] = d[u].y; dw[2] = d[u].z; dw[3] = d[u].w;
                        } else {
                            dw[0] = swap ? d[u].y : d[u].x; dw[1] = swap ? d[u].x : d[u].y; dw[2] = 0; dw[3] = 0;
                        }
#pragma unroll
                        for (int i = 0; i < NV; ++i) {
                            const uint32_t ioff = (V == 16) ? (uint32_t)(4 * i) * (uint32_t)sizeof(word) : (i ? step2 : 0u);
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const uint32_t b = __builtin_amdgcn_ubfe(dw[i], sh[k], 8u);
                                if (!SKIP || b != skipb[SKIP ? i : 0][k])
                                    Acc<W>::add(reinterpret_cast<word*>(lds_raw + (__umul24(b, pitch) + flk[k] + ioff)), v);
                            }
                        }
                    }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) { d[u] = dn[u]; gv[u] = gn[u]; }
                }
            }
            __syncthreads();
            if (cend >= gend) store_partial<W>(lds, plan.lds_bytes, slot);
            else merge_local<W>(lds, lds_words, ftp, ft, f0, F, hist, plan.hshift, plan.pad16 != 0);
        }
    }
}

// Contiguous rows with the whole row in one tile (16 <= F <= 64, F % 4 == 0, slice
// start 16-byte aligned): the rows of a chunk are one flat byte stream, read with
// 16-byte loads.  L lanes (16*L a multiple of F) cover RPI = 16*L/F whole rows per
// iteration, so a lane's four dwords keep their (row, feature) position for the
// whole kernel; they lie in at most two consecutive rows.  Blocks of U iterations
// are software-pipelined like in hist_kernel.
//
// TWO (32-bit working words only; 1024 threads, one workgroup per CU): a second copy of the local bins with 64-bit
// words (32|32 fields) sits next to the working copy; before the rows since the last fold exceed a chunk the working
// words are widened and added into it (every thread folds its own words: no atomics) and cleared, and the 64-bit copy
// is what the group hands over at its end.  A group may then be as long as its build allows -- one group per CU instead of one per chunk -- which
// for a build of all rows halves the bytes handed over and reduced, and no chunk is ever merged through global atomics.
template <int W, int U, bool TWO>
__global__ __launch_bounds__(TWO ? 1024 : HIST_THREADS, TWO ? 1 : HIST_WAVES) void hist_flat_kernel(RowSource src,
                                                         const HistEntry* __restrict__ entries,
                                                         const int32_t* __restrict__ table_counts,
                                                         int64_t* hist_base, unsigned char* partials, int F, int nb,
                                                         HistPlan plan, StepState* step) {
    using word = typename Acc<W>::word;
    extern __shared__ unsigned char lds_raw[];
    word* lds = reinterpret_cast<word*>(lds_raw);

    const int n_entries = table_counts[0], n_items = table_counts[1];
    const int hmul = (1 << (plan.hshift - 8)) - 1;
    if ((int)blockIdx.x >= n_items) return;
    if (step && blockIdx.x == 0 && threadIdx.x == 0) count_profile(entries, n_entries, false, step);

    const int RPI = plan.flat_rows, L = plan.flat_lanes;
    const int BR = U * RPI;  // rows of one block of U iterations
    const int ftp = plan.ftp;
    const int lds_words = nb * ftp;
    // (TWO) the 64-bit copy follows the working words, 16-byte aligned
    unsigned long long* lds2 = reinterpret_cast<unsigned long long*>(lds_raw + (((size_t)lds_words * sizeof(word) + 15) & ~(size_t)15));
    for (int w = threadIdx.x; w < lds_words; w += blockDim.x) lds[w] = 0;
    if (TWO)
        for (int w = threadIdx.x; w < lds_words; w += blockDim.x) lds2[w] = 0ull;
    __shared__ int s_start[TABLE_MAX];
    load_item_starts(entries, n_entries, s_start);

    const int lane0 = threadIdx.x & 63;
    const bool lane_on = lane0 < L;
    const int lane = lane_on ? lane0 : 0;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = blockDim.x >> 6;
    const uint32_t pitch = (uint32_t)ftp * (uint32_t)sizeof(word);
    // position of the lane's four dwords inside one iteration
    const int period = F / ((F % 16 == 0) ? 16 : (F % 8 == 0) ? 8 : 4);  // lanes after which the column repeats
    const int rot = lane / period;
    uint32_t sh[4], fl4[4][4];
    const int rA = (16 * lane) / F, rB = (16 * lane + 12) / F;
    bool useB[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int fo = 16 * lane + 4 * i;
        const int row = fo / F, col = fo - row * F;
        useB[i] = row != rA;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = (k + rot) & 3;
            if (i == 0) sh[k] = 8 * c;
            fl4[i][k] = (uint32_t)(col + c) * (uint32_t)sizeof(word);
        }
    }
    const int dpr = F / 4;
    const int align_rows = 16 / ((F % 16 == 0) ? 16 : (F % 8 == 0) ? 8 : 4);  // rows after which a row start is 16-byte aligned again
    // rows per chunk: whole blocks, and room for the unaligned head rows (fewer than align_rows) that the
    // first chunk of a build's first group takes on top, so that no local word sees more than chunk_rows rows
    const int chunk = (plan.chunk_rows - (align_rows - 1)) / BR * BR > 0 ? (plan.chunk_rows - (align_rows - 1)) / BR * BR : BR;

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const HistEntry en = entries[find_entry(s_start, n_entries, item)];
        const uint8_t* bins = src.bins[en.buf];
        const int16_t* gh = src.gh[en.buf];
        // the first rows up to a 16-byte aligned row start are taken by group 0, one dword at a time
        const int64_t head = min(en.count, (int64_t)((align_rows - (int)(en.begin % align_rows)) % align_rows));
        const int64_t body = en.count - head;
        int64_t rows_per_group = (body + en.groups - 1) / en.groups;
        rows_per_group = (rows_per_group + BR - 1) / BR * BR;  // keeps every group start 16-byte aligned
        if (rows_per_group < BR) rows_per_group = BR;
        const int g = item - en.item_start;
        const int64_t gbegin = min(en.count, head + (int64_t)g * rows_per_group);
        const int64_t gend = min(en.count, gbegin + rows_per_group);
        int64_t* hist = hist_base + (int64_t)en.slot * F * nb;
        unsigned char* slot = partials + (size_t)item * (size_t)plan.slot_bytes;
        bool first = true;  // a group without rows still hands over its (empty) bins

        if constexpr (TWO) {
            // One pass over the group's blocks, wavefront w taking blocks w, w + n_waves, ... in rounds that all
            // wavefronts walk together; after every `fold_rounds` rounds the working words are folded.  The loads of a
            // wavefront's next block stay in flight across a fold: only LDS is touched between the barriers.
            const uint8_t* cb = bins + (en.begin + gbegin) * (int64_t)F;
            const int16_t* gb = gh + (en.begin + gbegin);
            const int64_t grow = gend - gbegin;
            const int n_blocks = (int)(grow / BR);
            const int rounds = (n_blocks + n_waves - 1) / n_waves;
            // rows of `fold_rounds` rounds, plus the tail (< BR) and head (< align_rows) rows of the last period, fit a chunk
            const int fold_rounds = max(1, (plan.chunk_rows - BR - align_rows) / (n_waves * BR));
            auto fold = [&]() {
                __syncthreads();
                for (int w = threadIdx.x; w < lds_words; w += blockDim.x) {
                    const word v = lds[w];
                    if (v != 0) { lds[w] = 0; lds2[w] += (unsigned long long)Acc<W>::widen(v, plan.hshift); }
                }
                __syncthreads();
            };
            uint4 d[U], dn[U];
            int ga[U], gbv[U], gan[U], gbn[U];
            if (wave < n_blocks) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t row0 = (int64_t)(wave * U + u) * RPI;
                    d[u] = *reinterpret_cast<const uint4*>(cb + (size_t)row0 * (size_t)F + 16 * lane);
                    ga[u] = gb[row0 + rA];
                    gbv[u] = gb[row0 + rB];
                }
            }
            for (int r = 0; r < rounds; ++r) {
                const int jb = r * n_waves + wave;  // uniform over the wavefront
                if (jb < n_blocks) {
                    const int jn = min(jb + n_waves, n_blocks - 1);  // the last prefetch re-reads the last block
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int64_t row0 = (int64_t)(jn * U + u) * RPI;
                        dn[u] = *reinterpret_cast<const uint4*>(cb + (size_t)row0 * (size_t)F + 16 * lane);
                        gan[u] = gb[row0 + rA];
                        gbn[u] = gb[row0 + rB];
                    }
                    if (lane_on) {
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const word va = Acc<W>::expand(ga[u], hmul);
                            const word vb = Acc<W>::expand(gbv[u], hmul);
                            const uint32_t dw[4] = {d[u].x, d[u].y, d[u].z, d[u].w};
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const word v = useB[i] ? vb : va;
#pragma unroll
                                for (int k = 0; k < 4; ++k) {
                                    const uint32_t b = __builtin_amdgcn_ubfe(dw[i], sh[k], 8u);
                                    Acc<W>::add(reinterpret_cast<word*>(lds_raw + (__umul24(b, pitch) + fl4[i][k])), v);
                                }
                            }
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) { d[u] = dn[u]; ga[u] = gan[u]; gbv[u] = gbn[u]; }
                }
                if ((r + 1) % fold_rounds == 0 && r + 1 < rounds) fold();
            }
            // the rows after the last whole block and (group 0) the unaligned head rows in front of the
            // build: one dword per thread and step, into the last fold's rows
            const int64_t tail0 = (int64_t)n_blocks * BR;
            const int n_head = g == 0 ? (int)head : 0;
            const int n_tail = (int)(grow - tail0);
            for (int e = threadIdx.x; e < (n_head + n_tail) * dpr; e += blockDim.x) {
                const int rs = e / dpr, q = e - rs * dpr;
                const int64_t arow = rs < n_head ? (int64_t)rs : gbegin + tail0 + (rs - n_head);
                const uint32_t dwd = *reinterpret_cast<const uint32_t*>(bins + (en.begin + arow) * (int64_t)F + 4 * q);
                const word v = Acc<W>::expand(gh[en.begin + arow], hmul);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t b = (dwd >> (8 * k)) & 0xffu;
                    Acc<W>::add(&lds[b * ftp + 4 * q + k], v);
                }
            }
            fold();
            store_partial<32>(lds2, lds_words * 8, slot);
            __syncthreads();  // the next item's atomics wait for the cleared words
            continue;
        }

        for (int64_t cbegin = gbegin; first || cbegin < gend; cbegin += chunk) {
            const int64_t cend = min(gend, cbegin + (int64_t)chunk);
            const int crow = cbegin < cend ? (int)(cend - cbegin) : 0;
            __syncthreads();
            const uint8_t* cb = bins + (en.begin + cbegin) * (int64_t)F;
            const int16_t* gb = gh + (en.begin + cbegin);
            const int n_blocks = crow / BR;
            if (wave < n_blocks) {
                uint4 d[U], dn[U];
                int ga[U], gbv[U], gan[U], gbn[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int row0 = (wave * U + u) * RPI;
                    d[u] = *reinterpret_cast<const uint4*>(cb + (size_t)row0 * (size_t)F + 16 * lane);
                    ga[u] = gb[row0 + rA];
                    gbv[u] = gb[row0 + rB];
                }
                for (int jb = wave; jb < n_blocks; jb += n_waves) {
                    const int jn = min(jb + n_waves, n_blocks - 1);  // the last prefetch re-reads the last block
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int row0 = (jn * U + u) * RPI;  // uniform
                        dn[u] = *reinterpret_cast<const uint4*>(cb + (size_t)row0 * (size_t)F + 16 * lane);
                        gan[u] = gb[row0 + rA];
                        gbn[u] = gb[row0 + rB];
                    }
                    if (lane_on) {  // the lanes beyond the last whole row of an iteration sit out
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const word va = Acc<W>::expand(ga[u], hmul);
                        const word vb = Acc<W>::expand(gbv[u], hmul);
                        const uint32_t dw[4] = {d[u].x, d[u].y, d[u].z, d[u].w};
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const word v = useB[i] ? vb : va;
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const uint32_t b = __builtin_amdgcn_ubfe(dw[i], sh[k], 8u);
                                Acc<W>::add(reinterpret_cast<word*>(lds_raw + (__umul24(b, pitch) + fl4[i][k])), v);
                            }
                        }
                    }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) { d[u] = dn[u]; ga[u] = gan[u]; gbv[u] = gbn[u]; }
                }
            }
            // rows left over after the last whole block, and (first chunk of group 0) the unaligned
            // head rows in front of the group: one dword per thread and step
            const int tail0 = n_blocks * BR;
            const int n_head = (first && g == 0) ? (int)head : 0;
            const int n_tail = crow - tail0;
            for (int e = threadIdx.x; e < (n_head + n_tail) * dpr; e += blockDim.x) {
                const int rs = e / dpr, q = e - rs * dpr;
                // row index inside the entry: head rows come first, tail rows follow the chunk's blocks
                const int64_t arow = rs < n_head ? (int64_t)rs : cbegin + tail0 + (rs - n_head);
                const uint32_t dwd = *reinterpret_cast<const uint32_t*>(bins + (en.begin + arow) * (int64_t)F + 4 * q);
                const word v = Acc<W>::expand(gh[en.begin + arow], hmul);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t b = (dwd >> (8 * k)) & 0xffu;
                    Acc<W>::add(&lds[b * ftp + 4 * q + k], v);
                }
            }
            __syncthreads();
            if (cend >= gend) store_partial<W>(lds, plan.lds_bytes, slot);
            else merge_local<W>(lds, lds_words, ftp, F, 0, F, hist, plan.hshift);
            first = false;
        }
    }
}

// Any feature count and bin type (no alignment assumption): one load per (row, feature).  Serves 16-bit
// bins and rows or tiles narrower than a dword.  lane -> (row r of the iteration, feature f of the
// tile); a wavefront covers 64/C rows per iteration, C = the tile width rounded up to a power of two
// (tiles wider than 64 features are walked in steps of 64).
template <int W, typename BIN>
__global__ __launch_bounds__(HIST_THREADS) void hist_generic_kernel(RowSource src, IdxSet idxs, int use_idx,
                                                            const HistEntry* __restrict__ entries,
                                                            const int32_t* __restrict__ table_counts,
                                                            int64_t* hist_base, unsigned char* partials, int F,
                                                            int nb, HistPlan plan, StepState* step) {
    using word = typename Acc<W>::word;
    extern __shared__ unsigned char lds_raw[];
    word* lds = reinterpret_cast<word*>(lds_raw);
    const int n_entries = table_counts[0], n_items = table_counts[1];
    const int hmul = (1 << (plan.hshift - 8)) - 1;
    int tile, glane;
    tile_and_lane(plan.n_tiles, tile, glane);
    const int n_lanes = (int)gridDim.x / plan.n_tiles;
    if (glane >= n_items) return;
    if (step && blockIdx.x == 0 && threadIdx.x == 0) count_profile(entries, n_entries, use_idx != 0, step);
    const int f0 = tile * plan.ft;
    const int ft = min(plan.ft, F - f0);
    const int lds_words = ft * nb;
    for (int w = threadIdx.x; w < lds_words; w += blockDim.x) lds[w] = 0;
    __shared__ int s_start[TABLE_MAX];
    load_item_starts(entries, n_entries, s_start);
    int C = 1;
    while (C < ft && C < 64) C <<= 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    const int rpi = 64 / C;                  // rows per wavefront iteration
    const int r = lane / C, fl = lane % C;   // the lane's row of the iteration and first feature
    for (int item = glane; item < n_items; item += n_lanes) {
        const HistEntry en = entries[find_entry(s_start, n_entries, item)];
        const int64_t rows_per_group = (en.count + en.groups - 1) / en.groups;
        const int64_t gbegin = min(en.count, (int64_t)(item - en.item_start) * rows_per_group);
        const int64_t gend = min(en.count, gbegin + rows_per_group);
        int64_t* hist = hist_base + (int64_t)en.slot * F * nb;
        unsigned char* slot = partials + ((size_t)item * plan.n_tiles + tile) * (size_t)plan.slot_bytes;
        const int32_t* idx = use_idx ? (idxs.p[en.buf] + en.begin) : nullptr;
        const BIN* bins = reinterpret_cast<const BIN*>(src.bins[use_idx ? BUF_ORIGINAL : en.buf]);
        const bool gpos = use_idx && src.gh_pos != 0;
        const int16_t* gh = gpos ? src.gh[en.buf] + en.begin : src.gh[use_idx ? BUF_ORIGINAL : en.buf];
        for (int64_t cbegin = gbegin; cbegin < gend || cbegin == gbegin; cbegin += plan.chunk_rows) {
            const int64_t cend = min(gend, cbegin + (int64_t)plan.chunk_rows);
            __syncthreads();
            for (int64_t p = cbegin + wave * rpi + r; p < cend; p += n_waves * rpi) {
                const int64_t i = idx ? (int64_t)idx[p] : en.begin + p;
                const word v = Acc<W>::expand(gh[gpos ? p : i], hmul);
                const BIN* row = bins + i * F + f0;
                for (int f = fl; f < ft; f += C) Acc<W>::add(&lds[(uint32_t)row[f] * ft + f], v);
            }
            __syncthreads();
            if (cend >= gend) store_partial<W>(lds, lds_words * (int)sizeof(word), slot);
            else merge_local<W>(lds, lds_words, ft, ft, f0, F, hist, plan.hshift);
        }
    }
}

// Adds the slots of every build's row groups to the build's histogram.  Thread -> one word
// of a tile's local bins; the launch's items are cut into gridDim.z runs, a thread walks its
// run (consecutive items mostly belong to one build) and issues one 64-bit atomic per build
// it meets.  `generic` slots have the pitch of their tile's width, the others plan.ftp.
template <int W>
__global__ __launch_bounds__(256) void hist_reduce_kernel(const unsigned char* __restrict__ partials,
                                                          const HistEntry* __restrict__ entries,
                                                          const int32_t* __restrict__ table_counts,
                                                          int64_t* hist_base, int F, int nb, HistPlan plan,
                                                          int generic) {
    using word = typename Acc<W>::word;
    const int n_entries = table_counts[0], n_items = table_counts[1];
    const int hs = plan.hshift;
    const uint32_t hmask = (1u << hs) - 1u;
    const int per = (n_items + (int)gridDim.z - 1) / (int)gridDim.z;
    const int i0 = blockIdx.z * per, i1 = min(n_items, i0 + per);
    if (i0 >= i1) return;  // uniform over the workgroup
    __shared__ int s_start[TABLE_MAX];
    load_item_starts(entries, n_entries, s_start);
    const int f0 = blockIdx.y * plan.ft;
    const int ft = min(plan.ft, F - f0);
    const int pitch = generic ? ft : plan.ftp;
    const int w = blockIdx.x * blockDim.x + threadIdx.x;
    const int b = w / pitch;
    int f = w - b * pitch;
    if (!generic && plan.pad16) f = unpad16(f);
    if (b >= nb || f < 0 || f >= ft) return;
    const size_t stride = (size_t)gridDim.y * (size_t)plan.slot_bytes;  // bytes from one item's slot to the next
    const unsigned char* base = partials + (size_t)blockIdx.y * (size_t)plan.slot_bytes + (size_t)w * sizeof(word);
    const int64_t hoff = (int64_t)b * F + f0 + f;
    int e = find_entry(s_start, n_entries, i0);
    int i = i0;
    while (i < i1) {
        const int iend = min(i1, entries[e].item_start + entries[e].groups);
        int64_t sg = 0, sh = 0;
        for (; i + 4 <= iend; i += 4) {
            word v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] = *reinterpret_cast<const word*>(base + (size_t)(i + k) * stride);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (W == 16) { sg += (int32_t)v[k] >> hs; sh += (uint32_t)v[k] & hmask; }
                else sg += (int64_t)v[k];
            }
        }
        for (; i < iend; ++i) {
            const word v = *reinterpret_cast<const word*>(base + (size_t)i * stride);
            if (W == 16) { sg += (int32_t)v >> hs; sh += (uint32_t)v & hmask; }
            else sg += (int64_t)v;
        }
        const int64_t sum = (W == 16) ? sg * 4294967296LL + sh : sg;
        if (sum != 0)
            atomicAdd(reinterpret_cast<unsigned long long*>(hist_base + (int64_t)entries[e].slot * F * nb + hoff),
                      (unsigned long long)sum);
        ++e;
    }
}

static int64_t rows_fitting(int bits_g, int bits_h, int w) {
    const int64_t kg = (1 << (bits_g - 1)) - 1, kh = bits_h == 0 ? 1 : (1 << bits_h) - 2;  // bits_h 0: h~ = 1
    const int64_t a = (((int64_t)1 << (w - 1)) - 1) / kg;
    const int64_t b = (((int64_t)1 << w) - 1) / kh;
    return a < b ? a : b;
}

int64_t max_rows_for_width(int bits_g, int bits_h, int w) { return rows_fitting(bits_g, bits_h, w); }

// Rows a 32-bit local word takes when its low `s` bits hold the hessian sum (unsigned) and the
// 32 - s bits above it the gradient sum (signed); the s in 8..24 with the most rows, 16 on a tie.
static int64_t rows_fitting_word32(int bits_g, int bits_h, int* hshift) {
    const int64_t kg = (1 << (bits_g - 1)) - 1, kh = bits_h == 0 ? 1 : (1 << bits_h) - 2;
    int64_t best = -1;
    int bs = 16;
    for (int s = 8; s <= 24; ++s) {
        const int64_t a = (((int64_t)1 << (31 - s)) - 1) / kg;
        const int64_t b = (((int64_t)1 << s) - 1) / kh;
        const int64_t r = a < b ? a : b;
        if (r > best || (r == best && s == 16)) { best = r; bs = s; }
    }
    *hshift = bs;
    return best;
}

// Chooses tile width, accumulator width and launch shape for a problem shape.
HistPlan make_hist_plan(const qgbdt_shape& s, int bits_g, int bits_h, int acc_width, bool skew) {
    HistPlan p{};
    const int F = s.n_features, nb = s.n_bins;
    int hshift = 16;
    const int64_t n16 = rows_fitting_word32(bits_g, bits_h, &hshift);  // rows per chunk of 32-bit local words
    int w = acc_width;
    // a 16|16 chunk must amortise its hand-over: measured on 10.5 M x 28, whole trees, 16|16 against 32|32:
    // 4.07 / 4.17 ms at 4 bits (4681 rows per chunk), 4.29 / 4.10 ms at 5 bits (2184 rows)
    if (w == 0) w = (n16 >= 4096) ? 16 : 32;
    const int wbytes = (w == 16) ? 4 : 8;
    const int lds_budget = 64 * 1024;
    const int npd = 4 / s.bin_bytes;  // bins per dword
    const bool aligned = (F % npd == 0);
    // dword kernels: rows of any width >= 4 bytes (unaligned loads when not a multiple of 4 bytes)
    bool fast = aligned || F >= npd;
    int wide_ft = 0;
    if (!fast || s.bin_bytes != 1) {
    } else if (F % 16 == 0 && F > 64) {
        // wide rows: 16-byte pieces, padded local bins (20 words per 16 features)
        for (int ft = 256; ft >= 32 && !wide_ft; ft >>= 1)
            if ((int64_t)(ft + ft / 4) * nb * wbytes <= lds_budget) wide_ft = ft;
        if (wide_ft) { p.wide_v = 16; p.pad16 = 1; }
    } else if (F % 8 == 0 && F > 64) {
        // 8-byte pieces, at most 64 features per tile, unpadded
        // With 64-bit words and most-frequent-bin skipping, 64-feature tiles (130 KB of local bins, one workgroup
        // of 1024 threads per CU): whole 64-byte pieces of a row per lane group.  Without skipping the 64-bit
        // LDS atomics of such a tile cost more than its loads save (5M x 200: 577 against 476 us; with 70 % of
        // the entries skipped 373 us).
        const int budget8 = (skew && wbytes == 8) ? 136 * 1024 : lds_budget;
        for (int ft = 64; ft >= 32 && !wide_ft; ft >>= 1)
            if ((int64_t)ft * nb * wbytes <= budget8) wide_ft = ft;
        if (wide_ft) p.wide_v = 8;
    }
    if (wide_ft) {
        p.ft = wide_ft;
        p.ftp = p.pad16 ? wide_ft + wide_ft / 4 : wide_ft;
        p.dpr = wide_ft / 4;
        p.rows_per_it = 64 / p.dpr > 0 ? 64 / p.dpr : 1;
        p.lds_bytes = p.ftp * nb * wbytes;
    } else if (fast) {
        // candidates in order of preference: the whole row when it is narrow, then wide tiles
        // (whole cache lines per row), small tiles only when nothing else fits the LDS budget
        // (8-bit bins: tiles of at most 32 features get a pitch of 32 words, so that the LDS bank is the feature;
        // 16-bit bins have up to 1024 bin rows, a pitch of the tile width rounded up to 4 words lets wider tiles fit)
        const int cands[] = {(F <= 64) ? F : 0, 128, 96, 64, 48, 40, 32, 24, 16, 12, 8, 6, 4, 2};
        auto pitch_of = [&](int ft) { return (s.bin_bytes == 1 && ft <= 32) ? 32 : (ft + 3) / 4 * 4; };
        int best_ft = 0;
        for (int pass = 0; pass < 2 && best_ft == 0; ++pass) {
            double best_score = -1.0;
            for (int c = 0; c < 14; ++c) {
                const int ft = cands[c];
                if (ft <= 0 || ft > F || (ft % npd && ft != F)) continue;
                if (pass == 0 && ft < 32 && ft != F) continue;
                if ((int64_t)pitch_of(ft) * nb * wbytes > lds_budget) continue;
                const int dpr = (ft + npd - 1) / npd;
                if (dpr > 64) continue;
                const int rpi = 64 / dpr;
                const int tiles = (F + ft - 1) / ft;
                if (F - (tiles - 1) * ft < npd) continue;  // every tile row holds at least one dword
                const double score = ((double)(rpi * dpr) / 64.0) * ((double)F / ((double)tiles * ft));
                if (score > best_score + 1e-9) { best_score = score; best_ft = ft; }
            }
        }
        if (best_ft == 0 && aligned && (int64_t)pitch_of(npd) * nb * wbytes <= lds_budget) best_ft = npd;
        if (best_ft == 0) fast = false;
        p.ft = best_ft;
        p.ftp = pitch_of(best_ft > 0 ? best_ft : 1);
        p.dpr = (best_ft + npd - 1) / npd;
        p.rows_per_it = p.dpr > 0 ? 64 / p.dpr : 0;
        p.lds_bytes = p.ftp * nb * wbytes;
    }
    if (!wide_ft && !fast) {
        int ft = lds_budget / (nb * wbytes);
        if (ft > F) ft = F;
        if (ft < 1) ft = 1;
        p.ft = ft; p.ftp = ft; p.dpr = 0; p.rows_per_it = 0;
        p.lds_bytes = ft * nb * wbytes;
    }
    p.n_tiles = (F + p.ft - 1) / p.ft;
    const int64_t lim = (w == 16) ? n16 : rows_fitting(bits_g, bits_h, 32);
    p.chunk_rows = (int32_t)((lim > 0x40000000LL) ? 0x40000000LL : lim);
    if (p.chunk_rows < 1) p.chunk_rows = 1;
    p.min_rows_per_group = 2048;
    p.threads = (p.lds_bytes > 80 * 1024) ? 1024 : HIST_THREADS;
    int per_cu = (160 * 1024) / (p.lds_bytes > 0 ? p.lds_bytes : 1);
    // one-tile launches: the flat kernel needs ~100 VGPRs, so 16 wavefronts per CU are resident at once and
    // twice as many row groups would only double the slots to write and reduce; tiled launches measured
    // better with the groups of 32 wavefronts per CU
    int by_waves = (p.n_tiles == 1 ? 16 : 32) / (p.threads / 64);
    if (by_waves < 1) by_waves = 1;
    if (per_cu > by_waves) per_cu = by_waves;
    if (per_cu < 1) per_cu = 1;
    // Row-group lanes come in multiples of 8 (one per XCD).  One build (equal row groups, one per lane): rounded
    // down, so that all workgroups are resident at once -- 7 tiles at 2 workgroups per CU: 72 x 7 = 504 instead
    // of 80 x 7 = 560 workgroups for 512 places, whose last 48 would start when the first ones end (5 M x 200,
    // 64-bit words: 403 against 485 us).  Many builds of different sizes per launch: rounded up, the workgroups
    // end at different times anyway and the late ones fill in (20 M x 200: 13.06 against 13.13 ms per tree).
    int groups = (256 * per_cu) / p.n_tiles;
    if (groups < 1) groups = 1;
    p.max_lanes = (groups + 7) / 8 * 8;
    if (groups >= 8) groups = groups / 8 * 8;
    p.max_groups = groups;
    p.acc_width = w;
    p.hshift = hshift;
    p.ragged = (fast && !aligned) ? 1 : 0;
    p.bytewise = fast ? 0 : 1;
    p.flat_lanes = 0; p.flat_rows = 0;
    if (fast && aligned && s.bin_bytes == 1 && p.n_tiles == 1 && F >= 16 && F <= 64) {
        for (int l = 64; l >= 32; --l)
            if ((16 * l) % F == 0) { p.flat_lanes = l; p.flat_rows = 16 * l / F; break; }
    }
    p.flat_unroll = 2;
    p.slot_bytes = (p.lds_bytes + 15) & ~15;
    p.max_items = 4 * p.max_groups;
    if (p.max_items < 2 * s.max_leaves + 64) p.max_items = 2 * s.max_leaves + 64;
    p.single_rows = p.chunk_rows >= 1024 ? p.chunk_rows - 320 : p.chunk_rows / 2;
    if (p.single_rows < 1) p.single_rows = 1;
    return p;
}

// Plan for one build of `rows` rows.  With the width left open, 16|16 words are only taken when
// every row group can fit one chunk (the item table has room for rows / single_rows groups):
// beyond that groups would merge their earlier chunks through global atomics, which costs more
// than the 64-bit LDS atomics of 32|32 words (10.5 M rows, 5-bit: 236 us against 93 us).
//
// A long contiguous build (stream_ok) of a narrow matrix with 32-bit working words takes the byte-stream kernel's
// two-level form when every CU's group would span at least two chunks: 256 groups of 1024 threads, the working
// words folded into 64-bit words in LDS after every chunk.  With the width left open that needs chunks of at least
// 4096 rows (2- to 4-bit gradients), as for the one-level form.
HistPlan make_hist_plan_for(const qgbdt_shape& s, int bits_g, int bits_h, int acc_width, int64_t rows, bool skew,
                            bool stream_ok) {
    HistPlan p = make_hist_plan(s, bits_g, bits_h, acc_width, skew);
    if (stream_ok && acc_width != 32 && p.flat_lanes > 0) {
        HistPlan q = p.acc_width == 16 ? p : make_hist_plan(s, bits_g, bits_h, 16, skew);
        const int64_t words = (int64_t)s.n_bins * q.ftp;
        const int64_t lds = ((words * 4 + 15) & ~(int64_t)15) + words * 8;
        // one round of the 16 wavefronts (blocks of 2 iterations) plus a tail block and the head rows must fit a chunk
        const bool round_fits = q.chunk_rows >= 17 * 2 * q.flat_rows + 4;
        if ((acc_width == 16 || q.chunk_rows >= 4096) && round_fits && rows >= (int64_t)2 * 256 * q.chunk_rows &&
            lds <= 150 * 1024) {
            q.two_level = 1;
            q.threads = 1024;
            q.lds_bytes = (int32_t)lds;
            q.slot_bytes = (int32_t)((words * 8 + 15) & ~(int64_t)15);
            q.max_groups = 256;
            q.max_items = 256;  // one build, one group per CU
            q.max_lanes = 256;
            q.single_rows = 0x40000000;  // a group folds its chunks locally: no limit on its length
            return q;
        }
    }
    if (acc_width == 0 && p.acc_width == 16 && rows / p.single_rows >= (int64_t)p.max_items - 2)
        p = make_hist_plan(s, bits_g, bits_h, 32, skew);
    return p;
}

// One entry table for a stand-alone build.
__global__ void set_hist_table_kernel(HistEntry* entries, int32_t* counts, int64_t begin, int64_t count, HistPlan plan) {
    if (threadIdx.x == 0) {
        const int64_t t = hist_target_rows(plan, count, 1);
        int64_t g = (count + t - 1) / t;
        if (g < 1) g = 1;
        HistEntry e;
        e.begin = begin; e.count = count; e.buf = BUF_ORIGINAL; e.slot = 0; e.item_start = 0; e.groups = (int32_t)g;
        entries[0] = e;
        counts[0] = 1;
        counts[1] = count > 0 ? (int32_t)g : 0;
    }
}

int launch_set_hist_table(qgbdt_ctx* ctx, const HistPlan& plan, int64_t begin, int64_t count) {
    hipLaunchKernelGGL(set_hist_table_kernel, dim3(1), dim3(64), 0, ctx->stream, ctx->hist_entries, ctx->hist_counts,
                       begin, count, plan);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

// The wide-row kernels may be given more local bins than the default limit of dynamic LDS (the 64-feature tiles
// of 64-bit words that frequent-bin skipping makes worthwhile): the runtime is told so once per context.
template <int W, bool IDX, int V, bool S>
static hipError_t allow_lds(int bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(hist_wide_kernel<W, IDX, V, 4, S>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

int prepare_hist_kernels(qgbdt_ctx* ctx) {
    {
        // the two-level byte-stream kernel holds a 32-bit and a 64-bit copy of the local bins
        const HistPlan two = make_hist_plan_for(ctx->shape, 8, 8, 16, ctx->shape.n_rows, false, true);  // shortest chunks
        if (two.two_level && two.lds_bytes > 48 * 1024)
            QG_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(hist_flat_kernel<16, 2, true>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024));
    }
    int most = 0;
    for (int w = 16; w <= 32; w += 16)
        for (int skew = 0; skew < 2; ++skew) {
            const HistPlan hp = make_hist_plan(ctx->shape, 2, 2, w, skew != 0);
            if (hp.wide_v > 0 && hp.lds_bytes > most) most = hp.lds_bytes;
        }
    if (most <= 64 * 1024) return QGBDT_OK;
    QG_HIP(ctx, (allow_lds<16, false, 16, false>(most)));  QG_HIP(ctx, (allow_lds<16, false, 16, true>(most)));
    QG_HIP(ctx, (allow_lds<16, true, 16, false>(most)));   QG_HIP(ctx, (allow_lds<16, true, 16, true>(most)));
    QG_HIP(ctx, (allow_lds<16, false, 8, false>(most)));   QG_HIP(ctx, (allow_lds<16, false, 8, true>(most)));
    QG_HIP(ctx, (allow_lds<16, true, 8, false>(most)));    QG_HIP(ctx, (allow_lds<16, true, 8, true>(most)));
    QG_HIP(ctx, (allow_lds<32, false, 16, false>(most)));  QG_HIP(ctx, (allow_lds<32, false, 16, true>(most)));
    QG_HIP(ctx, (allow_lds<32, true, 16, false>(most)));   QG_HIP(ctx, (allow_lds<32, true, 16, true>(most)));
    QG_HIP(ctx, (allow_lds<32, false, 8, false>(most)));   QG_HIP(ctx, (allow_lds<32, false, 8, true>(most)));
    QG_HIP(ctx, (allow_lds<32, true, 8, false>(most)));    QG_HIP(ctx, (allow_lds<32, true, 8, true>(most)));
    return QGBDT_OK;
}

// Launches the kernel variant for (plan, row source).  `grid_items` is the host's upper bound on
// the number of work items; workgroups beyond the table's item count return at once.
int launch_hist(qgbdt_ctx* ctx, const HistPlan& plan, const RowSource& rows, const IdxSet& idx, bool use_idx,
                bool flat_ok, const HistEntry* entries, const int32_t* table_counts, int64_t* hist_base,
                int64_t grid_items, StepState* step, const uint16_t* mfb) {
    const int F = ctx->shape.n_features, nb = ctx->shape.n_bins;
    unsigned char* partials = static_cast<unsigned char*>(ctx->hist_partials);
    // The kernels address slot (item, tile) for item < max_items of the plan they are given (the tables they read
    // are built from the same plan and never hold more items): that range must lie inside the workspace's section,
    // and the flat grid must cut into whole XCD groups of row-group lanes.
    if ((size_t)plan.max_items * (size_t)plan.n_tiles * (size_t)plan.slot_bytes > ctx->hist_partials_bytes)
        return set_error(ctx, QGBDT_E_WORKSPACE,
                         "histogram plan needs %zu bytes of row-group slots (%d items x %d tiles x %d bytes), the workspace holds %zu",
                         (size_t)plan.max_items * plan.n_tiles * plan.slot_bytes, plan.max_items, plan.n_tiles,
                         plan.slot_bytes, ctx->hist_partials_bytes);
    if (plan.max_lanes % 8 != 0 || plan.max_lanes < 8 || plan.lds_bytes > 160 * 1024)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "inconsistent histogram plan (lanes %d, local bins %d bytes)", plan.max_lanes, plan.lds_bytes);
    int64_t groups = grid_items;
    if (groups > plan.max_lanes) groups = plan.max_lanes;
    if (groups < 1) groups = 1;
    // row-group lanes in multiples of 8 (one per XCD), times the feature tiles, as one flat grid
    const int64_t lanes = (groups + 7) / 8 * 8;
    dim3 grid((unsigned)(lanes * plan.n_tiles)), block(plan.threads);
    const bool fast = !plan.bytewise;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (ctx->profiling && ctx->ev_used + 2 <= ctx->ev_cap) {
        for (int k = 0; k < 2; ++k)
            if (!ctx->ev[ctx->ev_used + k]) QG_HIP(ctx, hipEventCreate(&ctx->ev[ctx->ev_used + k]));
        ctx->ev_root[ctx->ev_used / 2] = ctx->next_hist_is_root ? 1 : 0;
        e0 = ctx->ev[ctx->ev_used++]; e1 = ctx->ev[ctx->ev_used++];
        QG_HIP(ctx, hipEventRecord(e0, ctx->stream));
    }
    ctx->next_hist_is_root = 0;
    const bool flat = fast && !use_idx && plan.flat_lanes > 0 && flat_ok;
    if (plan.two_level && !flat)
        return set_error(ctx, QGBDT_E_INVALID_ARG, "two-level plan for rows that the byte-stream kernel cannot read");
    bool wide_ok = true;  // 16-byte loads need 16-byte aligned matrices (F is a multiple of 16 in that mode)
    for (int b = 0; b < 4; ++b) wide_ok = wide_ok && (((uintptr_t)rows.bins[b] & 15) == 0);
    if (flat) {
#define QG_LAUNCH_FLAT(W_, U_)                                                                                   \
    hipLaunchKernelGGL((hist_flat_kernel<W_, U_, false>), grid, block, plan.lds_bytes, ctx->stream, rows, entries, \
                       table_counts, hist_base, partials, F, nb, plan, step)
        if (plan.two_level) {
            hipLaunchKernelGGL((hist_flat_kernel<16, 2, true>), grid, block, plan.lds_bytes, ctx->stream, rows, entries,
                               table_counts, hist_base, partials, F, nb, plan, step);
        } else if (plan.acc_width == 16) {
            if (plan.flat_unroll >= 4) QG_LAUNCH_FLAT(16, 4);
            else if (plan.flat_unroll >= 2) QG_LAUNCH_FLAT(16, 2);
            else QG_LAUNCH_FLAT(16, 1);
        } else {
            if (plan.flat_unroll >= 4) QG_LAUNCH_FLAT(32, 4);
            else if (plan.flat_unroll >= 2) QG_LAUNCH_FLAT(32, 2);
            else QG_LAUNCH_FLAT(32, 1);
        }
#undef QG_LAUNCH_FLAT
    } else if (fast && plan.wide_v > 0 && wide_ok) {
#define QG_LAUNCH_WIDE_S(W_, IDX_, V_, U_, S_)                                                                        \
    do {                                                                                                              \
        hipLaunchKernelGGL((hist_wide_kernel<W_, IDX_, V_, U_, S_>), grid, block, plan.lds_bytes, ctx->stream, rows,  \
                           idx, entries, table_counts, hist_base, partials, F, nb, plan, step, mfb);                  \
    } while (0)
#define QG_LAUNCH_WIDE(W_, IDX_, V_, U_)                                                                              \
    do {                                                                                                              \
        if (mfb) QG_LAUNCH_WIDE_S(W_, IDX_, V_, U_, true); else QG_LAUNCH_WIDE_S(W_, IDX_, V_, U_, false);            \
    } while (0)
#define QG_LAUNCH_WIDE_V(W_, IDX_) \
    if (plan.wide_v == 16) QG_LAUNCH_WIDE(W_, IDX_, 16, 4); else QG_LAUNCH_WIDE(W_, IDX_, 8, 4)
        if (plan.acc_width == 16) {
            if (use_idx) { QG_LAUNCH_WIDE_V(16, true); } else { QG_LAUNCH_WIDE_V(16, false); }
        } else {
            if (use_idx) { QG_LAUNCH_WIDE_V(32, true); } else { QG_LAUNCH_WIDE_V(32, false); }
        }
#undef QG_LAUNCH_WIDE_V
#undef QG_LAUNCH_WIDE
#undef QG_LAUNCH_WIDE_S
    } else if (fast) {
        const int cap = 64 / plan.rows_per_it;
        const int U = cap >= 8 ? 8 : cap >= 7 ? 7 : cap >= 4 ? 4 : cap >= 2 ? 2 : 1;
#define QG_LAUNCH_HIST_K(W_, IDX_, U_, RAG_, BB_)                                                                  \
    hipLaunchKernelGGL((hist_kernel<W_, IDX_, U_, RAG_, BB_>), grid, block, plan.lds_bytes, ctx->stream, rows, idx,   \
                       entries, table_counts, hist_base, partials, F, nb, plan, step)
#define QG_LAUNCH_HIST(W_, IDX_, U_)                                                                               \
    do {                                                                                                           \
        if (ctx->shape.bin_bytes == 2) {                                                                           \
            if (plan.ragged) QG_LAUNCH_HIST_K(W_, IDX_, (U_ > 4 ? 4 : U_), true, 2);                               \
            else QG_LAUNCH_HIST_K(W_, IDX_, (U_ > 4 ? 4 : U_), false, 2);                                          \
        } else if (plan.ragged) QG_LAUNCH_HIST_K(W_, IDX_, (U_ > 4 ? 4 : U_), true, 1);                            \
        else QG_LAUNCH_HIST_K(W_, IDX_, U_, false, 1);                                                             \
    } while (0)
#define QG_LAUNCH_HIST_U(W_, IDX_)                                                      \
    switch (U) {                                                                        \
        case 8: QG_LAUNCH_HIST(W_, IDX_, 8); break;                                     \
        case 7: QG_LAUNCH_HIST(W_, IDX_, 7); break;                                     \
        case 4: QG_LAUNCH_HIST(W_, IDX_, 4); break;                                     \
        case 2: QG_LAUNCH_HIST(W_, IDX_, 2); break;                                     \
        default: QG_LAUNCH_HIST(W_, IDX_, 1); break;                                    \
    }
        if (plan.acc_width == 16) {
            if (use_idx) { QG_LAUNCH_HIST_U(16, true) } else { QG_LAUNCH_HIST_U(16, false) }
        } else {
            if (use_idx) { QG_LAUNCH_HIST_U(32, true) } else { QG_LAUNCH_HIST_U(32, false) }
        }
#undef QG_LAUNCH_HIST_U
#undef QG_LAUNCH_HIST
#undef QG_LAUNCH_HIST_K
    } else {
#define QG_LAUNCH_GENERIC(W_, BIN_)                                                                              \
    hipLaunchKernelGGL((hist_generic_kernel<W_, BIN_>), grid, block, plan.lds_bytes, ctx->stream, rows, idx, \
                       use_idx ? 1 : 0, entries, table_counts, hist_base, partials, F, nb, plan, step)
        if (ctx->shape.bin_bytes == 2) {
            if (plan.acc_width == 16) QG_LAUNCH_GENERIC(16, uint16_t); else QG_LAUNCH_GENERIC(32, uint16_t);
        } else {
            if (plan.acc_width == 16) QG_LAUNCH_GENERIC(16, uint8_t); else QG_LAUNCH_GENERIC(32, uint8_t);
        }
#undef QG_LAUNCH_GENERIC
    }
    QG_HIP(ctx, hipGetLastError());
    {
        // the slots of the row groups are added to the histograms
        const int tile_words = nb * (fast ? plan.ftp : plan.ft);
        const int xb = (tile_words + 255) / 256;
        int64_t items_bound = grid_items < plan.max_items ? grid_items : plan.max_items;
        int z = (int)(2048 / ((int64_t)xb * plan.n_tiles));
        if (z > 64) z = 64;
        if (z > items_bound) z = (int)items_bound;
        if (z < 1) z = 1;
        dim3 rgrid((unsigned)xb, (unsigned)plan.n_tiles, (unsigned)z);
        if (plan.acc_width == 16 && !plan.two_level)  // (two-level groups hand over 64-bit words)
            hipLaunchKernelGGL(hist_reduce_kernel<16>, rgrid, dim3(256), 0, ctx->stream, partials, entries, table_counts,
                               hist_base, F, nb, plan, fast ? 0 : 1);
        else
            hipLaunchKernelGGL(hist_reduce_kernel<32>, rgrid, dim3(256), 0, ctx->stream, partials, entries, table_counts,
                               hist_base, F, nb, plan, fast ? 0 : 1);
        QG_HIP(ctx, hipGetLastError());
    }
    if (e1) QG_HIP(ctx, hipEventRecord(e1, ctx->stream));
    return QGBDT_OK;
}

}  // namespace qgbdt
