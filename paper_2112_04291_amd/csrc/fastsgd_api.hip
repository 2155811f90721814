// C ABI of the gfx950 FastSGD codec: argument checks, workspace carve-up, kernel launches.
// Every entry point only enqueues work on the caller's stream.
#include <atomic>
#include <mutex>
#include <vector>

#include "fastsgd_device.hpp"
#include "fastsgd_encode_kernels.hpp"
#include "fastsgd_decode_kernels.hpp"

namespace fsgd {

#ifndef FSGD_AGG_TILE
#define FSGD_AGG_TILE 24576
#endif
constexpr u64 kDecSegBytes = 1152;   // >= sizeof(DecSeg)
constexpr u32 kMaxSegments = 65536;
constexpr u32 kInlineWaves = 16;       // waves per workgroup of a single-stream decode launch over a long stream ...
constexpr u64 kInlineLargeBytes = 6u << 20;   // ... which is one of at least this many bytes (some 3000 key blocks)
constexpr u64 kMaxElems = 0xFFFFFFFFull - 1023;   // per gradient: scratch offsets inside a segment stay below 2^32
constexpr u32 kMaxSumGrid = 2048;      // most workgroups the abs-sum pass of a single gradient is launched with
static_assert(sizeof(DecSeg) <= kDecSegBytes, "decoder workspace records");
static_assert(sizeof(SegInfo) == 48 && sizeof(SegBatch) <= 3900, "segment table travels as a kernel argument");

static bool params_ok(const fastsgd_params* p) {
    if (!p) return false;
    if (!(p->base >= 1.0 + 1.0 / 1048576.0) || !(p->base <= 16.0)) return false;
    if (p->tau < 1 || p->tau > kMaxTau) return false;
    if (p->tau > 128 && !(p->base <= 4.0)) return false;       // b^tau stays finite (and sum / b^c a normal binary64)
    if (p->flag_bits < 1 || p->flag_bits > 5) return false;
    if (p->block_keys < 256 || p->block_keys > kMaxKB || (p->block_keys & (p->block_keys - 1))) return false;
    return p->reserved == 0;
}

static u64 up(u64 x, u64 a) { return (x + a - 1) / a * a; }

// Workspace layout from bounds that depend only on (total_n, n_segments, min_block_keys), so the size
// query and the call agree.
static EncodePlan make_plan(u64 total_n, u32 n_segments, u32 min_kb) {
    EncodePlan pl{};
    pl.total_n = total_n;
    pl.n_segments = n_segments;
    pl.n_slots = (n_segments == 1) ? kMaxSumGrid : 4u;           // abs-sum records per segment
    pl.max_items = total_n / min_kb + n_segments + 1;              // bound on key blocks (+1 per empty segment)
    pl.max_slots = total_n + 4ull * n_segments + 8;                // scratch entries: element index + 4 per segment
    pl.max_rows = total_n / kRow + 2ull * n_segments + 2;           // a segment adds at most two partial rows
    // about kChunkTarget chunks, more only where that would make a chunk longer than kMaxChunkRows; a
    // segment adds at most one short chunk
    const u64 by_length = pl.max_rows / kMaxChunkRows + 1;
    pl.max_chunks = (by_length > kChunkTarget ? by_length : (u64)kChunkTarget) + n_segments;
    u64 o = 0;
    pl.off_ctrl = o;  o += up(sizeof(Ctrl), 256);
    pl.off_gsum = o;  o += up((u64)(kMaxGroups + 1) * 8, 256);
    pl.zero_end = o;                                               // a single-gradient call clears up to here
    pl.off_gbins = o; o += up((u64)n_segments * pl.n_slots * kBinWords * 8, 256);
    pl.zero_end_batch = o;                                         // a batch also clears the abs-sum records
    pl.off_rowmax = o;   o += up((pl.max_rows + kTile / kRow) * 2 * kRowGranules, 256);   // a 16-bit bound per granule (+ a tile)
    pl.off_ccount = o;   o += up(pl.max_chunks * 4, 256);
    pl.off_binfo = o;    o += up(pl.max_items * sizeof(BlockInfo), 256);
    pl.off_seginfo = o;  o += up((u64)n_segments * sizeof(SegInfo), 256);
    pl.off_segstate = o; o += up((u64)n_segments * sizeof(SegState), 256);
    pl.off_skeys = o;    o += up(pl.max_slots * 4, 256);
    pl.off_scodes = o;                                             // last: a byte per code, ...
    pl.total_narrow = o + up(pl.max_slots, 256);
    pl.total = o + up(pl.max_slots * 2, 256);                      // ... 16 bits when some tau is above 128
    return pl;
}

static u32 cu_count() {
    static std::atomic<u32> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    u32 c = cached[dev].load(std::memory_order_relaxed);
    if (c == 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        c = (u32)v;
        cached[dev].store(c, std::memory_order_relaxed);
    }
    return c;
}

// Optional per-kernel timing for the profiling entry points: events recorded on the launch stream
// before the first kernel and after every kernel.
struct Marks {
    hipEvent_t* ev = nullptr;
    u32 next = 0;
    void mark(hipStream_t s) { if (ev) (void)hipEventRecord(ev[next++], s); }
};

static u32 clamp_grid(u64 want, u64 cap) { u64 g = want < cap ? want : cap; return (u32)(g ? g : 1); }

static fastsgd_status compress_impl(const u32* d_keys, const float* d_values, const u64* seg_offsets, u32 n_segments,
                                    const fastsgd_params* params, u32 params_stride, void* d_out, size_t out_capacity,
                                    u64* d_out_offsets, u32* d_status, void* d_ws, size_t ws_bytes, void* hip_stream,
                                    bool single, Marks marks = Marks()) {
    if (!seg_offsets || !params || !d_out || !d_out_offsets || !d_status || !d_ws) return FASTSGD_ERR_INVALID_ARG;
    if (n_segments < 1 || n_segments > kMaxSegments || params_stride > 1) return FASTSGD_ERR_INVALID_ARG;
    if (((uintptr_t)d_out & 7) || ((uintptr_t)d_ws & 255) || ((uintptr_t)d_values & 3) || ((uintptr_t)d_keys & 3))
        return FASTSGD_ERR_INVALID_ARG;
    const u64 first_elem = seg_offsets[0];
    const u64 total_n = seg_offsets[n_segments] - first_elem;
    if (seg_offsets[n_segments] < first_elem || total_n >= (1ull << 40)) return FASTSGD_ERR_INVALID_ARG;
    if (total_n && !d_values) return FASTSGD_ERR_INVALID_ARG;

    // elements are counted from the 16-byte boundary at or below the first one; keys keep their pairing
    const u64 mis = total_n ? ((uintptr_t)(d_values + first_elem) & 15) / 4 : 0;
    const float* vbase = d_values + first_elem - mis;
    const u32* kbase = d_keys ? d_keys + first_elem - mis : nullptr;     // no key array: keys are 0..n-1

    SegInfo one_seg;                                               // a single gradient needs no heap
    std::vector<SegInfo> seg_table;
    if (n_segments > 1) seg_table.resize(n_segments);
    SegInfo* segs = n_segments > 1 ? seg_table.data() : &one_seg;
    u32 min_kb = kMaxKB, max_kb = 0;
    bool wide = false;                                             // some segment's codes need more than a byte
    u64 n_tiles = 0, max_items = 0, total_rows = 0;
    for (u32 s = 0; s < n_segments; ++s) {
        const fastsgd_params* p = &params[params_stride ? s : 0];
        if (!params_ok(p)) return FASTSGD_ERR_INVALID_ARG;
        if (seg_offsets[s + 1] < seg_offsets[s]) return FASTSGD_ERR_INVALID_ARG;
        const u64 cnt = seg_offsets[s + 1] - seg_offsets[s];
        if (cnt > kMaxElems) return FASTSGD_ERR_INVALID_ARG;
        SegInfo& si = segs[s];
        si.elem_begin = seg_offsets[s] - first_elem + mis;
        si.elem_count = cnt;
        si.base = p->base; si.tau = p->tau; si.flag_bits = p->flag_bits; si.block_keys = p->block_keys;
        if (n_tiles >= 0xFFFFFFFFull) return FASTSGD_ERR_INVALID_ARG;
        si.tile_begin = (u32)n_tiles;
        const u64 span = cnt ? si.elem_begin + cnt - (si.elem_begin & ~3ull) : 0;   // from the aligned start
        n_tiles += (span + kTile - 1) / kTile;
        si.row_begin = (u32)total_rows;
        total_rows += (span + kRow - 1) / kRow;
        const u64 blocks = (cnt + p->block_keys - 1) / p->block_keys;
        max_items += blocks ? blocks : 1;
        if (p->block_keys < min_kb) min_kb = p->block_keys;
        if (p->block_keys > max_kb) max_kb = p->block_keys;
        if (p->tau > 128) wide = true;
    }
    // chunks of R rows, about kChunkTarget of them, never shorter than one tile
    u64 R64 = (total_rows + kChunkTarget - 1) / kChunkTarget;
    if (R64 < 2 * kValRows) R64 = 2 * kValRows;
    // a batch: whole batches of rows per chunk, so that no chunk ends on a batch of a row or two (a single
    // gradient's chunks are long enough for that not to matter, and more chunks serve it better)
    if (n_segments > 1) R64 = (R64 + kValRows - 1) / kValRows * kValRows;
    if (R64 > kMaxChunkRows) R64 = kMaxChunkRows;                  // (a multiple of kValRows)
    u64 n_chunks = 0;
    for (u32 s = 0; s < n_segments; ++s) {
        SegInfo& si = segs[s];
        const u64 span = si.elem_count ? si.elem_begin + si.elem_count - (si.elem_begin & ~3ull) : 0;
        const u64 rows = (span + kRow - 1) / kRow;
        si.chunk_begin = (u32)n_chunks;
        const u64 c = (rows + R64 - 1) / R64;
        if (c > kMaxSegChunks) return FASTSGD_ERR_INVALID_ARG;     // cannot happen: a gradient has under 2^24 + 2 rows
        n_chunks += c;
    }
    const EncodePlan pl = make_plan(total_n, n_segments, min_kb);
    if (total_rows > pl.max_rows || total_rows >= 0xFFFFFFFFull) return FASTSGD_ERR_INVALID_ARG;
    if (n_chunks > pl.max_chunks || max_items > pl.max_items || n_tiles >= 0xFFFFFFFFull)
        return FASTSGD_ERR_INVALID_ARG;
    if (ws_bytes < (wide ? pl.total : pl.total_narrow)) return FASTSGD_ERR_BUFFER_TOO_SMALL;
    if (out_capacity < kHeaderBytes) return FASTSGD_ERR_BUFFER_TOO_SMALL;
    const u32 R = (u32)R64;
    u32 g_shift = 6;                                               // key blocks per group of the size sums
    while ((pl.max_items >> g_shift) + 1 > kMaxGroups) ++g_shift;

    uint8_t* ws = static_cast<uint8_t*>(d_ws);
    Ctrl* ctrl = reinterpret_cast<Ctrl*>(ws + pl.off_ctrl);
    unsigned long long* gsum = reinterpret_cast<unsigned long long*>(ws + pl.off_gsum);
    u64* gbins = reinterpret_cast<u64*>(ws + pl.off_gbins);
    uint16_t* rowmax = reinterpret_cast<uint16_t*>(ws + pl.off_rowmax);
    u32* ccount = reinterpret_cast<u32*>(ws + pl.off_ccount);
    BlockInfo* binfo = reinterpret_cast<BlockInfo*>(ws + pl.off_binfo);
    SegInfo* dsegs = reinterpret_cast<SegInfo*>(ws + pl.off_seginfo);
    SegState* dstates = reinterpret_cast<SegState*>(ws + pl.off_segstate);
    u32* skeys = reinterpret_cast<u32*>(ws + pl.off_skeys);
    uint8_t* scodes = ws + pl.off_scodes;
    uint8_t* out = static_cast<uint8_t*>(d_out);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const u32 cus = cu_count();

    marks.mark(stream);
    const u64 zero_words = ((single ? pl.zero_end : pl.zero_end_batch) - pl.off_ctrl) / 8;
    u64* zero_begin = reinterpret_cast<u64*>(ws + pl.off_ctrl);
    if (!single) {
        // clear control words, counters and abs-sum records; store the segment table (kSegBatch per launch)
        for (u32 first = 0; first < n_segments; first += kSegBatch) {
            SegBatch b;
            const u32 count = (n_segments - first < kSegBatch) ? n_segments - first : kSegBatch;
            for (u32 i = 0; i < count; ++i) b.seg[i] = segs[first + i];
            if (first == 0)
                hipLaunchKernelGGL(k_init, dim3(clamp_grid((zero_words + 1023) / 1024, 2048)), dim3(256), 0, stream,
                                   zero_begin, zero_words, dsegs, b, first, count);
            else
                hipLaunchKernelGGL(k_store_segments, dim3(1), dim3(128), 0, stream, dsegs, b, first, count);
        }
    }

    // (three workgroups per compute unit: four fit and run 2 % slower, two 17 %, six to eight with shared accumulators 6 %)
    u32 sum_grid = cus * 3 < kMaxSumGrid ? cus * 3 : kMaxSumGrid;
    sum_grid = clamp_grid(n_tiles, sum_grid);
    if (single)
        hipLaunchKernelGGL(k_abs_sum<true>, dim3(sum_grid), dim3(kThreads), 0, stream, vbase, dsegs, 1u, n_tiles,
                           gbins, sum_grid, zero_begin, zero_words, segs[0], dsegs, rowmax);
    else
        hipLaunchKernelGGL(k_abs_sum<false>, dim3(sum_grid), dim3(kThreads), 0, stream, vbase, dsegs, n_segments,
                           n_tiles, gbins, pl.n_slots, zero_begin, (u64)0, segs[0], dsegs, rowmax);
    marks.mark(stream);
    hipLaunchKernelGGL(k_tables, dim3(n_segments), dim3(kTableThreads), 0, stream, dsegs, dstates, gbins,
                       single ? sum_grid : pl.n_slots, ctrl);
    marks.mark(stream);
    if (n_chunks) {
        const dim3 grid((u32)((n_chunks + kValWaves - 1) / kValWaves)), block(kValWaves * kWave);
        if (wide)
            hipLaunchKernelGGL(k_encode_values<true>, grid, block, 0, stream, kbase, vbase, dsegs, dstates, n_segments,
                               (u32)n_chunks, R, rowmax, ccount, skeys, (void*)scodes);
        else
            hipLaunchKernelGGL(k_encode_values<false>, grid, block, 0, stream, kbase, vbase, dsegs, dstates, n_segments,
                               (u32)n_chunks, R, rowmax, ccount, skeys, (void*)scodes);
    }
    marks.mark(stream);
    hipLaunchKernelGGL(k_plan_segments, dim3(n_segments), dim3(kThreads), 0, stream, dsegs, dstates, n_segments, R,
                       ccount, ctrl);
    if (n_segments > 1)
        hipLaunchKernelGGL(k_number_segments, dim3(1), dim3(kThreads), 0, stream, dstates, n_segments, ctrl);
    const u64 max_units = (max_items + kWaves - 1) / kWaves + n_segments;
    if (max_kb > kSub)
        hipLaunchKernelGGL(k_measure_keys<true>, dim3(clamp_grid(max_units, (u64)cus * 4)), dim3(kThreads), 0, stream,
                           segs[0], dsegs, dstates, n_segments, R, ccount, skeys, binfo, gsum, g_shift, ctrl);
    else
        hipLaunchKernelGGL(k_measure_keys<false>, dim3(clamp_grid(max_units, (u64)cus * 8)), dim3(kThreads), 0, stream,
                           segs[0], dsegs, dstates, n_segments, R, ccount, skeys, binfo, gsum, g_shift, ctrl);
    marks.mark(stream);
    if (wide)
        hipLaunchKernelGGL(k_pack_keys<true>, dim3(clamp_grid(max_units, (u64)cus * 4)), dim3(kThreads), 0, stream, segs[0],
                           dsegs, dstates, n_segments, R, ccount, skeys, (const void*)scodes, binfo, gsum, g_shift, out,
                           (u64)out_capacity, d_out_offsets, single ? 1u : 0u, d_status, ctrl);
    else
        hipLaunchKernelGGL(k_pack_keys<false>, dim3(clamp_grid(max_units, (u64)cus * 4)), dim3(kThreads), 0, stream, segs[0],
                           dsegs, dstates, n_segments, R, ccount, skeys, (const void*)scodes, binfo, gsum, g_shift, out,
                           (u64)out_capacity, d_out_offsets, single ? 1u : 0u, d_status, ctrl);
    marks.mark(stream);
    return hipGetLastError() == hipSuccess ? FASTSGD_OK : FASTSGD_ERR_DEVICE;
}

static fastsgd_status decompress_impl(const void* d_streams, size_t total_bytes, const u64* d_stream_offsets,
                                      u32 n_segments, u32* d_keys_out, float* d_values_out, u64 capacity,
                                      u64* d_counts, u32* d_status, void* d_ws, size_t ws_bytes, void* hip_stream,
                                      bool single, Marks marks = Marks()) {
    if (!d_streams || !d_counts || !d_status || !d_ws) return FASTSGD_ERR_INVALID_ARG;
    if (n_segments < 1 || n_segments > kMaxSegments) return FASTSGD_ERR_INVALID_ARG;
    if (!single && !d_stream_offsets) return FASTSGD_ERR_INVALID_ARG;
    if (((uintptr_t)d_streams & 7) || ((uintptr_t)d_ws & 255)) return FASTSGD_ERR_INVALID_ARG;
    if (capacity && (!d_keys_out || !d_values_out)) return FASTSGD_ERR_INVALID_ARG;
    if (((uintptr_t)d_keys_out & 3) || ((uintptr_t)d_values_out & 3)) return FASTSGD_ERR_INVALID_ARG;
    if (ws_bytes < kDecSegOffset + (u64)n_segments * kDecSegBytes) return FASTSGD_ERR_BUFFER_TOO_SMALL;
    uint8_t* ws = static_cast<uint8_t*>(d_ws);
    DecCtrl* ctrl = reinterpret_cast<DecCtrl*>(ws);
    DecSeg* segs = reinterpret_cast<DecSeg*>(ws + kDecSegOffset);
    const uint8_t* streams = static_cast<const uint8_t*>(d_streams);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const u32 cus = cu_count();

    marks.mark(stream);
    // every key costs at least three bits, so bytes/96 bounds the number of key blocks
    const u64 max_blocks = (u64)total_bytes / 96 + n_segments;
    const u32 grid = clamp_grid((max_blocks + kWaves - 1) / kWaves, (u64)cus * 7);
    if (single) {
        // One launch: every workgroup checks the header and rebuilds the magnitude table itself.  A long
        // stream (thousands of key blocks: every wave slot of the GPU busy) is decoded by one large workgroup
        // per compute unit, so that one walk of b^c serves sixteen waves; a short one by small workgroups,
        // which spread its few blocks over more compute units.
        DecDone* done = reinterpret_cast<DecDone*>(ws + kDecDoneOffset);
        if (total_bytes >= kInlineLargeBytes)
            hipLaunchKernelGGL((k_decode<kStore, true, kInlineWaves>), dim3(clamp_grid((max_blocks + kInlineWaves - 1) / kInlineWaves, cus)),
                               dim3(kInlineWaves * kWave), 0, stream, streams, (u64)total_bytes, capacity, (const DecSeg*)nullptr, 1u,
                               ctrl, done, d_keys_out, d_values_out, d_counts, 1u, d_status, (float*)nullptr, (u64)0, 0u, AdamArgs());
        else
            hipLaunchKernelGGL((k_decode<kStore, true, kWaves>), dim3(clamp_grid((max_blocks + kWaves - 1) / kWaves, (u64)cus * 4)),
                               dim3(kThreads), 0, stream, streams, (u64)total_bytes, capacity, (const DecSeg*)nullptr, 1u,
                               ctrl, done, d_keys_out, d_values_out, d_counts, 1u, d_status, (float*)nullptr, (u64)0, 0u, AdamArgs());
    } else {
        hipLaunchKernelGGL(k_decode_clear, dim3(1), dim3(64), 0, stream, ctrl);
        hipLaunchKernelGGL(k_decode_setup, dim3(n_segments), dim3(kMaxTau), 0, stream, streams, (u64)total_bytes,
                           d_stream_offsets, n_segments == 1 ? 1u : 0u, segs, ctrl, capacity, d_counts, d_status);
        if (n_segments > 1)
            hipLaunchKernelGGL(k_decode_plan, dim3(1), dim3(kThreads), 0, stream, segs, n_segments, capacity, ctrl,
                               d_counts, d_status, (u64*)nullptr);
        hipLaunchKernelGGL((k_decode<kStore, false, kWaves>), dim3(grid), dim3(kThreads), 0, stream, streams, (u64)total_bytes, capacity,
                           segs, n_segments, ctrl, (DecDone*)nullptr, d_keys_out, d_values_out, d_counts, n_segments + 1u, d_status,
                           (float*)nullptr, (u64)0, 0u, AdamArgs());
    }
    marks.mark(stream);
    return hipGetLastError() == hipSuccess ? FASTSGD_OK : FASTSGD_ERR_DEVICE;
}

// Decode-and-aggregate: the streams are checked and planned like a batch; then either one launch per stream
// adds that stream's values into the dense array (sparse streams), or one launch per group of eight streams
// takes the dense array through shared memory once (dense streams).  Either way the additions at a key
// happen stream after stream.
static fastsgd_status accumulate_impl(const void* d_streams, size_t total_bytes, const u64* d_stream_offsets,
                                      u32 n_streams, float* d_dense, u64 dense_len, u64* d_count, u32* d_status,
                                      void* d_ws, size_t ws_bytes, void* hip_stream) {
    if (!d_streams || !d_count || !d_status || !d_ws || !d_stream_offsets) return FASTSGD_ERR_INVALID_ARG;
    if (n_streams < 1 || n_streams > kMaxSegments) return FASTSGD_ERR_INVALID_ARG;
    if (((uintptr_t)d_streams & 7) || ((uintptr_t)d_ws & 255) || ((uintptr_t)d_dense & 3)) return FASTSGD_ERR_INVALID_ARG;
    if (dense_len && !d_dense) return FASTSGD_ERR_INVALID_ARG;
    const u64 off_counts = kDecSegOffset + up((u64)n_streams * kDecSegBytes, 256);
    if (ws_bytes < off_counts + ((u64)n_streams + 1) * 8) return FASTSGD_ERR_BUFFER_TOO_SMALL;
    uint8_t* ws = static_cast<uint8_t*>(d_ws);
    DecCtrl* ctrl = reinterpret_cast<DecCtrl*>(ws);
    DecSeg* segs = reinterpret_cast<DecSeg*>(ws + kDecSegOffset);
    u64* counts = reinterpret_cast<u64*>(ws + off_counts);
    const uint8_t* streams = static_cast<const uint8_t*>(d_streams);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const u32 cus = cu_count();
    hipLaunchKernelGGL(k_decode_clear, dim3(1), dim3(64), 0, stream, ctrl);
    hipLaunchKernelGGL(k_decode_setup, dim3(n_streams), dim3(kMaxTau), 0, stream, streams, (u64)total_bytes,
                       d_stream_offsets, 0u, segs, ctrl, ~0ull, counts, d_status);
    hipLaunchKernelGGL(k_decode_plan, dim3(1), dim3(kThreads), 0, stream, segs, n_streams, ~0ull, ctrl, counts, d_status,
                       d_count);
    // Gradients that keep more than a few in a thousand of their entries: one pass over the dense vector per
    // group of streams instead of one per stream.  A pair of the other form moves two 64-byte lines of the dense
    // vector through the memory system (read and write back) for some two or three bytes of stream; the pass
    // moves eight bytes per entry of the vector for each group.  Measured on a 124 M vector with eight streams,
    // the pass wins from about one kept entry in two hundred on: ten stream bytes per entry of the vector and
    // group.  (The streams' pair counts are on the device only; their bytes are what the host can go by.)
    const u64 n_groups = ((u64)n_streams + kTileStreams - 1) / kTileStreams;
    const bool by_tiles = n_streams >= 2 && dense_len >= 1 && ((uintptr_t)d_dense & 15) == 0 &&
                          (u64)total_bytes * 10 >= dense_len * n_groups;
    if (by_tiles) {
        // a workgroup per compute unit, each with a run of tiles of its own (short vectors: runs of three, so
        // that few tiles do not mean as many workgroups that each start every stream afresh)
        constexpr u32 kTile = FSGD_AGG_TILE;
        const u64 n_tiles = (dense_len + kTile - 1) / kTile;
        const u64 groups = cus;
        u64 per = (n_tiles + groups - 1) / groups;
        if (per < 3) per = n_tiles < 3 ? n_tiles : 3;
        const u32 grid = (u32)((n_tiles + per - 1) / per);
        for (u32 s0 = 0; s0 < n_streams; s0 += kTileStreams) {
            const u32 n_here = n_streams - s0 < kTileStreams ? n_streams - s0 : kTileStreams;
            hipLaunchKernelGGL((k_accumulate_tiles<kTile>), dim3(grid), dim3(kTileStreams * kWave), 0, stream, streams, segs,
                               s0, n_here, ctrl, d_count, d_status, d_dense, dense_len, (u32)per);
        }
        return hipGetLastError() == hipSuccess ? FASTSGD_OK : FASTSGD_ERR_DEVICE;
    }
    const u32 grid = clamp_grid(((u64)total_bytes / 96 + 1 + kWaves - 1) / kWaves, (u64)cus * 7);
    for (u32 s = 0; s < n_streams; ++s)
        hipLaunchKernelGGL((k_decode<kAccum, false, kWaves>), dim3(grid), dim3(kThreads), 0, stream, streams, (u64)total_bytes, ~0ull,
                           segs, n_streams, ctrl, (DecDone*)nullptr, (u32*)nullptr, (float*)nullptr, d_count, 1u, d_status, d_dense, dense_len, s,
                           AdamArgs());
    return hipGetLastError() == hipSuccess ? FASTSGD_OK : FASTSGD_ERR_DEVICE;
}

// Decode-and-update: one stream, the Adam step of Section 4.1 at its keys.
static fastsgd_status adam_impl(const void* d_stream, size_t stream_bytes, float* d_theta, float* d_m, float* d_v,
                                u64 dim, const fastsgd_adam* h, u64* d_count, u32* d_status, void* d_ws,
                                size_t ws_bytes, void* hip_stream) {
    if (!d_stream || !d_count || !d_status || !d_ws || !h) return FASTSGD_ERR_INVALID_ARG;
    if (((uintptr_t)d_stream & 7) || ((uintptr_t)d_ws & 255)) return FASTSGD_ERR_INVALID_ARG;
    if (((uintptr_t)d_theta & 3) || ((uintptr_t)d_m & 3) || ((uintptr_t)d_v & 3)) return FASTSGD_ERR_INVALID_ARG;
    if (dim && (!d_theta || !d_m || !d_v)) return FASTSGD_ERR_INVALID_ARG;
    if (!(h->eta == h->eta) || !(h->beta1 >= 0.0 && h->beta1 <= 1.0) || !(h->beta2 >= 0.0 && h->beta2 <= 1.0) ||
        !(h->eps >= 0.0))
        return FASTSGD_ERR_INVALID_ARG;
    if (ws_bytes < kDecSegOffset + kDecSegBytes) return FASTSGD_ERR_BUFFER_TOO_SMALL;
    uint8_t* ws = static_cast<uint8_t*>(d_ws);
    DecCtrl* ctrl = reinterpret_cast<DecCtrl*>(ws);
    DecSeg* segs = reinterpret_cast<DecSeg*>(ws + kDecSegOffset);
    const uint8_t* streams = static_cast<const uint8_t*>(d_stream);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    AdamArgs a;
    a.m = d_m;
    a.v = d_v;
    a.eta = (float)h->eta;
    a.beta1 = (float)h->beta1;
    a.one_minus_beta1 = (float)(1.0 - h->beta1);
    a.beta2 = (float)h->beta2;
    a.one_minus_beta2 = (float)(1.0 - h->beta2);
    a.eps = (float)h->eps;
    // (two launches: with the header work inside it this variant of the decode kernel runs out of registers)
    hipLaunchKernelGGL(k_decode_setup, dim3(1), dim3(kMaxTau), 0, stream, streams, (u64)stream_bytes, (const u64*)nullptr, 1u,
                       segs, ctrl, ~0ull, d_count, d_status);
    const u32 grid = clamp_grid(((u64)stream_bytes / 96 + 1 + kWaves - 1) / kWaves, (u64)cu_count() * 7);
    hipLaunchKernelGGL((k_decode<kAdam, false, kWaves>), dim3(grid), dim3(kThreads), 0, stream, streams, (u64)stream_bytes, ~0ull,
                       segs, 1u, ctrl, (DecDone*)nullptr, (u32*)nullptr, (float*)nullptr, d_count, 1u, d_status, d_theta, dim, 0u, a);
    return hipGetLastError() == hipSuccess ? FASTSGD_OK : FASTSGD_ERR_DEVICE;
}

// Streaming read probe: 16 bytes per lane (non-temporal loads); a workgroup takes 16 KB at a time (four loads
// per lane in flight),
// consecutive workgroups take consecutive pieces; the data only feeds a hash that decides a store that
// (practically) never happens.
__global__ void __launch_bounds__(kThreads) k_probe_read(const uint4* __restrict__ src, u64 n16, u64* sink) {
    constexpr u32 U = 4;
    const u64 stride = (u64)gridDim.x * kThreads * U;
    u32 h = 0;
    for (u64 base = (u64)blockIdx.x * kThreads * U + threadIdx.x; base < n16; base += stride) {
        uint4 q[U];
#pragma unroll
        for (u32 r = 0; r < U; ++r) {
            const u64 i = base + r * kThreads;
            q[r] = i < n16 ? load_stream16(src + i) : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (u32 r = 0; r < U; ++r) h ^= q[r].x ^ q[r].y ^ q[r].z ^ q[r].w;
    }
    if (h == 0x9E3779B9u && __popcll(__ballot(true)) == 1) sink[0] = h;
}

// Runs `call` `iterations` times with an event after every kernel and averages the gaps.
template <class Call>
static fastsgd_status profile_loop(u32 n_kernels, u32 iterations, float* kernel_ms, hipStream_t stream, Call call) {
    if (!kernel_ms || iterations < 1 || iterations > 4096) return FASTSGD_ERR_INVALID_ARG;
    const u32 per = n_kernels + 1;
    std::vector<hipEvent_t> ev((size_t)per * iterations);
    for (auto& e : ev)
        if (hipEventCreate(&e) != hipSuccess) return FASTSGD_ERR_DEVICE;
    fastsgd_status rc = FASTSGD_OK;
    for (u32 it = 0; it < iterations && rc == FASTSGD_OK; ++it) {
        Marks m;
        m.ev = ev.data() + (size_t)it * per;
        rc = call(m);
    }
    if (hipStreamSynchronize(stream) != hipSuccess) rc = FASTSGD_ERR_DEVICE;
    for (u32 k = 0; k < n_kernels; ++k) kernel_ms[k] = 0.f;
    if (rc == FASTSGD_OK) {
        for (u32 it = 0; it < iterations; ++it)
            for (u32 k = 0; k < n_kernels; ++k) {
                float ms = 0.f;
                (void)hipEventElapsedTime(&ms, ev[(size_t)it * per + k], ev[(size_t)it * per + k + 1]);
                kernel_ms[k] += ms / (float)iterations;
            }
    }
    for (auto& e : ev) (void)hipEventDestroy(e);
    return rc;
}

}  // namespace fsgd

// Workspace of fastsgd_compress_static: one array per GPU the library runs on, held until the process
// ends.  Host code never uses the array's name as an address: the device address is looked up once per
// device (static_scratch) and passed to the kernels like any caller's workspace.
static __device__ __align__(256) unsigned char scratch[FASTSGD_STATIC_SCRATCH_BYTES];

namespace fsgd {

static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[64];                                    // per device, nullptr until looked up

// Device address of `scratch` on the current device, or nullptr (unknown device, lookup failed).
static void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace fsgd

using namespace fsgd;

extern "C" {

size_t fastsgd_compressed_size(uint64_t n, const fastsgd_params* p) {
    if (!params_ok(p) || n > kMaxElems) return 0;
    const u64 KB = p->block_keys, nb = (n + KB - 1) / KB;
    const u64 per_block = 8 * ((KB * p->flag_bits + 63) / 64 + (KB * 32 + 63) / 64);
    u32 width = 1;                                       // 1 + ceil(log2 tau) bits per value token
    while ((1u << (width - 1)) < p->tau) ++width;
    return (size_t)(kHeaderBytes + 8 * ((n * width + 63) / 64) + 16 * nb + nb * per_block);
}

size_t fastsgd_workspace_size(uint64_t total_n, uint32_t n_segments, uint32_t min_block_keys) {
    if (n_segments < 1 || n_segments > kMaxSegments || total_n >= (1ull << 40)) return 0;
    if (min_block_keys < 256 || min_block_keys > kMaxKB || (min_block_keys & (min_block_keys - 1))) return 0;
    // (the plan's bounds leave room for the call shifting its base down to a 16-byte boundary: 8 scratch entries
    // and two rows beyond the elements)
    return (size_t)make_plan(total_n, n_segments, min_block_keys).total;
}

size_t fastsgd_workspace_size_tau(uint64_t total_n, uint32_t n_segments, uint32_t min_block_keys, uint32_t max_tau) {
    if (n_segments < 1 || n_segments > kMaxSegments || total_n >= (1ull << 40)) return 0;
    if (min_block_keys < 256 || min_block_keys > kMaxKB || (min_block_keys & (min_block_keys - 1))) return 0;
    if (max_tau < 1 || max_tau > kMaxTau) return 0;
    const EncodePlan pl = make_plan(total_n, n_segments, min_block_keys);
    return (size_t)(max_tau > 128 ? pl.total : pl.total_narrow);
}

size_t fastsgd_decompress_workspace_size(uint32_t n_segments) {
    if (n_segments < 1 || n_segments > kMaxSegments) return 0;
    return (size_t)(kDecSegOffset + up((u64)n_segments * kDecSegBytes, 256) + ((u64)n_segments + 1) * 8);
}

fastsgd_status fastsgd_decompress_accumulate(const void* d_streams, size_t total_bytes,
                                             const uint64_t* d_stream_offsets, uint32_t n_streams, float* d_dense,
                                             uint64_t dense_len, uint64_t* d_count, uint32_t* d_status,
                                             void* d_workspace, size_t workspace_bytes, void* hip_stream) {
    return accumulate_impl(d_streams, total_bytes, d_stream_offsets, n_streams, d_dense, dense_len, d_count, d_status,
                           d_workspace, workspace_bytes, hip_stream);
}

fastsgd_status fastsgd_decompress_adam(const void* d_stream, size_t stream_bytes, float* d_theta, float* d_m, float* d_v,
                                       uint64_t dim, const fastsgd_adam* h, uint64_t* d_count, uint32_t* d_status,
                                       void* d_workspace, size_t workspace_bytes, void* hip_stream) {
    return adam_impl(d_stream, stream_bytes, d_theta, d_m, d_v, dim, h, d_count, d_status, d_workspace, workspace_bytes,
                     hip_stream);
}

fastsgd_status fastsgd_compress(const uint32_t* d_keys, const float* d_values, uint64_t n, const fastsgd_params* p,
                                void* d_out, size_t out_capacity, uint64_t* d_out_bytes, uint32_t* d_status,
                                void* d_workspace, size_t workspace_bytes, void* hip_stream) {
    if (n > kMaxElems) return FASTSGD_ERR_INVALID_ARG;
    const u64 offs[2] = {0, n};
    return compress_impl(d_keys, d_values, offs, 1, p, 0, d_out, out_capacity, d_out_bytes, d_status, d_workspace,
                         workspace_bytes, hip_stream, true);
}

fastsgd_status fastsgd_compress_static(const uint32_t* d_keys, const float* d_values, uint64_t n,
                                       const fastsgd_params* p, void* d_out, size_t out_capacity,
                                       uint64_t* d_out_bytes, uint32_t* d_status, void* hip_stream) {
    if (n > FASTSGD_STATIC_MAX_ELEMS) return FASTSGD_ERR_BUFFER_TOO_SMALL;      // beyond what the fixed workspace holds
    if (!params_ok(p)) return FASTSGD_ERR_INVALID_ARG;
    if (make_plan(FASTSGD_STATIC_MAX_ELEMS, 1, 256).total > FASTSGD_STATIC_SCRATCH_BYTES) return FASTSGD_ERR_DEVICE;
    void* ws = static_scratch();
    if (!ws) return FASTSGD_ERR_DEVICE;
    const u64 offs[2] = {0, n};
    return compress_impl(d_keys, d_values, offs, 1, p, 0, d_out, out_capacity, d_out_bytes, d_status, ws,
                         FASTSGD_STATIC_SCRATCH_BYTES, hip_stream, true);
}

fastsgd_status fastsgd_profile_compress(const uint32_t* d_keys, const float* d_values, uint64_t n,
                                        const fastsgd_params* p, void* d_out, size_t out_capacity,
                                        uint64_t* d_out_bytes, uint32_t* d_status, void* d_workspace,
                                        size_t workspace_bytes, void* hip_stream, uint32_t iterations,
                                        float* kernel_ms) {
    if (n > kMaxElems) return FASTSGD_ERR_INVALID_ARG;
    const u64 offs[2] = {0, n};
    return profile_loop(FASTSGD_PROFILE_COMPRESS_KERNELS, iterations, kernel_ms, static_cast<hipStream_t>(hip_stream),
                        [&](Marks m) {
                            return compress_impl(d_keys, d_values, offs, 1, p, 0, d_out, out_capacity, d_out_bytes,
                                                 d_status, d_workspace, workspace_bytes, hip_stream, true, m);
                        });
}

fastsgd_status fastsgd_probe_read(const void* d_src, size_t bytes, uint64_t* d_sink, void* hip_stream) {
    if (!d_src || !d_sink || ((uintptr_t)d_src & 15)) return FASTSGD_ERR_INVALID_ARG;
    const u64 n16 = bytes / 16;
    const u32 grid = clamp_grid((n16 + kThreads - 1) / kThreads, (u64)cu_count() * 8);
    hipLaunchKernelGGL(k_probe_read, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const uint4*>(d_src), n16, (u64*)d_sink);
    return hipGetLastError() == hipSuccess ? FASTSGD_OK : FASTSGD_ERR_DEVICE;
}

fastsgd_status fastsgd_profile_decompress(const void* d_stream, size_t stream_bytes, uint32_t* d_keys_out,
                                          float* d_values_out, uint64_t capacity, uint64_t* d_count,
                                          uint32_t* d_status, void* d_workspace, size_t workspace_bytes,
                                          void* hip_stream, uint32_t iterations, float* kernel_ms) {
    return profile_loop(FASTSGD_PROFILE_DECOMPRESS_KERNELS, iterations, kernel_ms,
                        static_cast<hipStream_t>(hip_stream), [&](Marks m) {
                            return decompress_impl(d_stream, stream_bytes, nullptr, 1, d_keys_out, d_values_out,
                                                   capacity, d_count, d_status, d_workspace, workspace_bytes,
                                                   hip_stream, true, m);
                        });
}

fastsgd_status fastsgd_compress_segmented(const uint32_t* d_keys, const float* d_values, const uint64_t* seg_offsets,
                                          uint32_t n_segments, const fastsgd_params* params, uint32_t params_stride,
                                          void* d_out, size_t out_capacity, uint64_t* d_out_seg_offsets,
                                          uint32_t* d_status, void* d_workspace, size_t workspace_bytes,
                                          void* hip_stream) {
    return compress_impl(d_keys, d_values, seg_offsets, n_segments, params, params_stride, d_out, out_capacity,
                         d_out_seg_offsets, d_status, d_workspace, workspace_bytes, hip_stream, false);
}

fastsgd_status fastsgd_decompress(const void* d_stream, size_t stream_bytes, uint32_t* d_keys_out, float* d_values_out,
                                  uint64_t capacity, uint64_t* d_count, uint32_t* d_status, void* d_workspace,
                                  size_t workspace_bytes, void* hip_stream) {
    return decompress_impl(d_stream, stream_bytes, nullptr, 1, d_keys_out, d_values_out, capacity, d_count, d_status,
                           d_workspace, workspace_bytes, hip_stream, true);
}

fastsgd_status fastsgd_decompress_segmented(const void* d_streams, size_t total_bytes, const uint64_t* d_stream_offsets,
                                            uint32_t n_segments, uint32_t* d_keys_out, float* d_values_out,
                                            uint64_t capacity, uint64_t* d_pair_offsets, uint32_t* d_status,
                                            void* d_workspace, size_t workspace_bytes, void* hip_stream) {
    return decompress_impl(d_streams, total_bytes, d_stream_offsets, n_segments, d_keys_out, d_values_out, capacity,
                           d_pair_offsets, d_status, d_workspace, workspace_bytes, hip_stream, false);
}

}  // extern "C"
