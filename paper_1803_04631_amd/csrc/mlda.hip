// libmlda.so: C ABI, context and host-side preprocessing (see include/mlda.h).
//
// Paper sections behind the host steps: Section 6.1.2 (tokens are sorted word-first and
// the tokens of heavy words are split over several workgroups), Section 6.2 (a
// document->token map lets the theta update find a document's tokens in the word-sorted
// arrays; the paper builds it on the CPU, here it is derived on the device), Section 4 and Algorithm 1 (the corpus is partitioned by document
// into chunks; WorkSchedule1: one chunk, transferred once, iterated on the device;
// WorkSchedule2: several chunks per GPU, transferred every iteration while phi stays).
//
// A context is the model (phi, n_k, tables) plus the chunk that is attached at the moment:
// with one chunk it is attached once and for all, with several each is attached in turn.
#include "../../include/mlda.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "kernels_rebuild.hpp"
#include "kernels_sample.hpp"

namespace {

thread_local std::string g_last_error;

int fail(int code, const std::string& msg) {
    g_last_error = msg;
    return code;
}

#define HIP_TRY(expr)                                                                  \
    do {                                                                               \
        hipError_t e_ = (expr);                                                        \
        if (e_ != hipSuccess)                                                          \
            return fail(MLDA_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    } while (0)

#define RC_TRY(expr)                   \
    do {                               \
        const int rc_ = (expr);        \
        if (rc_ != MLDA_OK) return rc_; \
    } while (0)

constexpr size_t kAlign = 256;        // workspace sub-buffer alignment
constexpr size_t kSlotAlign = 64;     // theta row slot alignment (bytes)
// waves per sampling workgroup: more of them share one staged p* column when K is large
// (twelve: two such workgroups fill a CU's six waves per SIMD, and their LDS fits twice)
int sample_waves_for(int32_t K) { return K <= 2048 ? 4 : 12; }

// theta rows with 2-byte entries where the topics fit their ten bits
bool tiny_rows_for(int32_t K) { return K <= mlda::TinyRows::kMaxK; }

// What the sampler's LDS holds besides p* itself belongs to K as well: Kpad = K + 1 rounded up to
// a multiple of the dense bucket's group (one zero entry of p* past the last topic: padding
// entries of theta rows point at it).
int32_t kpad_for(int32_t K) {
    const int32_t g = mlda::dense_group(sample_waves_for(K));
    return (K + g) / g * g;
}
// p* of one word beside the prefix sums and the waves' records: where that exceeds the LDS a
// workgroup can have on this chip (K beyond about 30,900), p* lives in device memory instead,
// one strip per workgroup of a launch of at most kFarStrips workgroups.
constexpr size_t kLdsPerWorkgroup = 160 * 1024;
constexpr int kFarStrips = 512;
bool far_weights_for(int32_t K) {
    return mlda::sample_lds_bytes(kpad_for(K), sample_waves_for(K)) > kLdsPerWorkgroup;
}

// short_docs: no document has more tokens than a 4-byte entry counts; near: the theta slots of
// the chunk end below 4 GiB, so that 32-bit byte offsets reach them
template <bool kNear>
const void* sample_kernel_of(int32_t K, bool short_docs) {
    if (far_weights_for(K)) return (const void*)mlda::sample_kernel<12, mlda::PackedRows, true, kNear>;
    if (tiny_rows_for(K)) return (const void*)mlda::sample_kernel<4, mlda::TinyRows, false, kNear>;
    if (sample_waves_for(K) == 4)
        return short_docs ? (const void*)mlda::sample_kernel<4, mlda::PackedRowsShort, false, kNear>
                          : (const void*)mlda::sample_kernel<4, mlda::PackedRows, false, kNear>;
    return short_docs ? (const void*)mlda::sample_kernel<12, mlda::PackedRowsShort, false, kNear>
                      : (const void*)mlda::sample_kernel<12, mlda::PackedRows, false, kNear>;
}
const void* sample_kernel_for(int32_t K, bool short_docs, bool near) {
    return near ? sample_kernel_of<true>(K, short_docs) : sample_kernel_of<false>(K, short_docs);
}
bool slots_near(size_t slots_bytes) { return slots_bytes <= 0xffffffffull; }
const void* theta_kernel_for(bool tiny, bool wide_counters) {
    if (tiny) return wide_counters ? (const void*)mlda::theta_rows_kernel<mlda::TinyRows, true>
                                   : (const void*)mlda::theta_rows_kernel<mlda::TinyRows, false>;
    return wide_counters ? (const void*)mlda::theta_rows_kernel<mlda::PackedRows, true>
                         : (const void*)mlda::theta_rows_kernel<mlda::PackedRows, false>;
}
constexpr int kMaxTimedIters = 1024;
constexpr int kRunTiles = 16;           // small tiles a workgroup of the large-K sampler takes one after the other
// events of a streamed chunk visit: its uploads have arrived | topics and slots in word-major
// order | theta rebuilt | sampled | phi added to | new topics in document order | theta of the
// new topics (log-likelihood)
constexpr int kVisitEvents = 7;
constexpr int kMaxTimedVisits = 4096;

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int tile_tokens_for(int32_t K) { return K <= 2048 ? 1024 : 4096; }
constexpr int kPhiSegment = 16384;    // tokens one workgroup histograms for the phi rebuild
constexpr int32_t kHistTopics = 32768; // 32-bit counters of the phi and n_k histograms that share a workgroup's LDS

// A theta row's slot: a header of kRowHeader bytes (the row's number of entries), then the
// entries, filled up to whole 16-byte units.  A document of n tokens needs at most
// min(n, K + n / max_count) entries: one per topic, and one more for every max_count tokens
// that a count exceeds its entry's field by.
size_t slot_bytes_for(int64_t n, int32_t K, int entry_bytes, int max_count) {
    const int64_t cap = std::min<int64_t>(n, (int64_t)K + n / max_count);
    return align_up((size_t)mlda::kRowHeader + align_up((size_t)cap * (size_t)entry_bytes, 16), kSlotAlign);
}

constexpr int kLoglikBlocks = 2048;
constexpr int kMaxThetaGrid = 8192;    // workgroups of the theta rebuild (each leaves one likelihood partial)
constexpr int kEntryRing = 2048;      // per-rebuild counters of theta row entries (> kMaxTimedIters)

// Where the buffers of one chunk of documents lie inside its part of the workspace (byte
// offsets).  The static part (up to static_bytes) is the preprocessed corpus and is copied
// from the host as one block; two index arrays derived from it on the device, z and the theta
// rows follow.
struct ChunkLayout {
    size_t tok_slot = 0, tok_id = 0, doc_map = 0, doc_ptr = 0, doc_order = 0, row_rec = 0, tiles = 0,
           segs = 0, split = 0, static_bytes = 0, doc_pairs = 0, z0 = 0, z1 = 0, slots = 0, total = 0;
};

// `streamed`: the chunk takes turns on the device with others.  It then needs no
// document->token map: its assignments arrive in document order (z_doc, in the map's place) and
// are paired with their documents' slots there (doc_pairs) on their way to word-major order.
ChunkLayout chunk_layout(int64_t D, int64_t T, size_t slots_bytes, size_t n_tiles, size_t n_segs,
                         size_t n_split, bool streamed) {
    ChunkLayout L;
    size_t at = 0;
    auto put = [&](size_t bytes) { const size_t o = at; at += align_up(bytes, kAlign); return o; };
    L.tok_id = put((size_t)T * 4);
    L.doc_ptr = put((size_t)(D + 1) * 4);
    L.doc_order = put((size_t)D * sizeof(mlda::DocRec));
    L.row_rec = put((size_t)D * 8);
    L.tiles = put(n_tiles * sizeof(mlda::Tile));
    L.segs = put(n_segs * sizeof(mlda::Tile));
    L.split = put(n_split * 4);
    L.static_bytes = at;
    L.tok_slot = put((size_t)T * 4);       // derived on the device from the static part
    L.doc_map = put((size_t)T * (streamed ? 2 : 4));
    L.doc_pairs = put(streamed ? (size_t)T * 8 : 0);
    L.z0 = put((size_t)T * 2);
    L.z1 = put((size_t)T * 2);
    L.slots = put(slots_bytes);
    L.total = at;
    return L;
}

// An upper bound of the same from the sizes alone.
ChunkLayout chunk_layout_bound(int64_t D, int64_t T, int32_t V, int32_t K, bool streamed) {
    const size_t tile = (size_t)tile_tokens_for(K);
    // (at most one entry of at most 4 bytes per token, a header, a unit's and a slot's rounding)
    const size_t slots = kSlotAlign + (size_t)T * 4 + (size_t)D * (mlda::kRowHeader + 16 + kSlotAlign);
    const size_t n_tiles = (size_t)T / tile + (size_t)V + 1;
    const size_t n_segs = (size_t)T / kPhiSegment + (size_t)V + 1;
    return chunk_layout(D, T, slots, n_tiles, n_segs, (size_t)V, streamed);
}

// The model and the scratch of the reductions.
// phi[i] is one copy of the model: the 16-bit matrix [V][K], then room for the int32 rows of
// the words with 2^16 tokens or more, of which a corpus of T tokens has at most T / 2^16.
struct ModelLayout {
    size_t phi[2] = {0, 0}, phi_wide = 0, phi_bytes = 0, wide_row = 0, n_k[2] = {0, 0}, ll_partial = 0,
           ll_scalars = 0, lg_table = 0, row_entries = 0, far_pstar = 0, total = 0;
};

int64_t wide_rows_bound(int32_t V, int64_t T) {
    return std::min<int64_t>((int64_t)V, T / mlda::kNarrowWordLimit);
}

ModelLayout model_layout(int32_t V, int32_t K, int64_t T, bool two_phi) {
    ModelLayout L;
    size_t at = 0;
    auto put = [&](size_t bytes) { const size_t o = at; at += align_up(bytes, kAlign); return o; };
    L.phi_wide = align_up((size_t)V * (size_t)K * 2, kAlign);      // offset of the wide rows inside a copy
    L.phi_bytes = L.phi_wide + align_up((size_t)wide_rows_bound(V, T) * (size_t)K * 4, kAlign);
    L.phi[0] = put(L.phi_bytes);
    L.phi[1] = two_phi ? put(L.phi_bytes) : L.phi[0];
    L.wide_row = put((size_t)V * 4);
    L.n_k[0] = put((size_t)K * 4);
    L.n_k[1] = two_phi ? put((size_t)K * 4) : L.n_k[0];
    L.ll_partial = put((size_t)(2 * kLoglikBlocks + kMaxThetaGrid) * 8);
    L.ll_scalars = put(4 * 8);                            // value, theta sum, document term, spare
    L.lg_table = put((size_t)(mlda::kLgTable + 1) * 8 * 2);   // one for alpha, one for beta
    L.row_entries = put((size_t)kEntryRing * 8);
    L.far_pstar = put(far_weights_for(K) ? (size_t)kFarStrips * (size_t)kpad_for(K) * 4 : 0);
    L.total = at;
    return L;
}

// body(0) .. body(n_chunks - 1), each on a thread of its own.  Nothing escapes a thread: an
// exception inside a part (host memory running out) is caught there, every thread that was
// started is joined, and the call returns false.  Parts whose thread could not be started
// run on the calling thread.
template <class F>
bool parallel_chunks(int n_chunks, F&& body) {
    std::vector<std::thread> pool;
    std::vector<char> failed((size_t)std::max(n_chunks, 1), 0);
    auto guarded = [&](int c) {
        try { body(c); } catch (...) { failed[(size_t)c] = 1; }
    };
    int started = 1;
    try {
        pool.reserve((size_t)std::max(n_chunks - 1, 0));
        for (; started < n_chunks; ++started) pool.emplace_back(guarded, started);
    } catch (...) {
        // no more threads (or no memory for them): the rest runs here, below
    }
    guarded(0);
    for (int c = started; c < n_chunks; ++c) guarded(c);
    for (auto& t : pool) t.join();
    for (char f : failed)
        if (f) return false;
    return true;
}

// Documents [d_begin, d_end) of the corpus, preprocessed: the static part of the chunk's
// buffers, laid out as on the device.
struct HostChunk {
    int64_t d_begin = 0, d_end = 0;
    int64_t tok_begin = 0;              // caller's index of the chunk's first token
    int64_t D = 0, T = 0;
    bool tiny = false;                  // theta rows as 2-byte entries (K < 1024), else 4-byte
    bool wide_counters = false;         // some document has 2^16 tokens or more
    bool short_docs = true;             // no document has more tokens than a 4-byte entry counts
    size_t slots_bytes = 0;
    int32_t n_tiles = 0, n_segs = 0, n_split = 0;
    int32_t n_single = 0;               // the tiles from this one on hold whole small words: taken in runs
    int64_t run_tokens = 0;             // their tokens
    int32_t n_wide_tiles = 0;           // sampling tiles of words whose row of phi is int32
    ChunkLayout L;
    unsigned char* arena = nullptr;     // L.static_bytes bytes
    bool pinned = false;

    HostChunk() = default;
    HostChunk(const HostChunk&) = delete;
    HostChunk& operator=(const HostChunk&) = delete;
    ~HostChunk() { release(); }
    void release() {
        if (arena) {
            if (pinned) (void)hipHostFree(arena); else std::free(arena);
            arena = nullptr;
        }
    }
};

// Word-first order (Section 6.1.2), document->token map (Section 6.2), theta row slots, tiles.
// Inside a word the tokens are put in order of falling document length, so that the theta
// rows a wave walks together have similar lengths; any order inside a word gives the same
// result, because the uniforms are keyed by the caller's token index.  `accumulate`: the
// chunk's counts will be added to phi (several chunks) instead of stored.
int prepare_chunk(const int64_t* doc_ptr_all, const int32_t* word_ids_all, int64_t d_begin,
                  int64_t d_end, int32_t V, int32_t K, bool accumulate, bool pinned, bool runs, HostChunk& h) {
    const int64_t D = d_end - d_begin;
    const int64_t tok_begin = doc_ptr_all[d_begin];
    const int64_t T = doc_ptr_all[d_end] - tok_begin;
    const int32_t* word_ids = word_ids_all ? word_ids_all + tok_begin : nullptr;
    auto len_of = [&](int64_t d) { return doc_ptr_all[d_begin + d + 1] - doc_ptr_all[d_begin + d]; };
    auto start_of = [&](int64_t d) { return doc_ptr_all[d_begin + d] - tok_begin; };
    h.d_begin = d_begin; h.d_end = d_end; h.tok_begin = tok_begin; h.D = D; h.T = T;

    int64_t longest_doc = 0;
    for (int64_t d = 0; d < D; ++d) longest_doc = std::max(longest_doc, len_of(d));
    h.tiny = tiny_rows_for(K);
    // a count never exceeds the document's length: 16-bit counters in the theta rebuild if
    // they hold it
    h.wide_counters = longest_doc >= 65536;
    h.short_docs = longest_doc <= mlda::PackedRows::kMaxCount;
    const int entry_bytes = h.tiny ? mlda::TinyRows::kEntryBytes : mlda::PackedRows::kEntryBytes;
    const int max_count = h.tiny ? mlda::TinyRows::kMaxCount : mlda::PackedRows::kMaxCount;

    std::vector<int32_t> doc_order;              // documents by falling length
    std::vector<int64_t> order_tokens;           // tokens before each position of doc_order
    std::vector<uint32_t> slot_of;               // slot offset of each document, 16-byte units
    std::vector<int32_t> word_ptr;
    try {
        doc_order.resize((size_t)D);
        order_tokens.resize((size_t)D + 1);
        std::vector<int64_t> len_start((size_t)longest_doc + 2, 0);
        for (int64_t d = 0; d < D; ++d) ++len_start[(size_t)(longest_doc - len_of(d)) + 1];
        for (int64_t l = 0; l <= longest_doc; ++l) len_start[(size_t)l + 1] += len_start[(size_t)l];
        for (int64_t d = 0; d < D; ++d) doc_order[(size_t)len_start[(size_t)(longest_doc - len_of(d))]++] = (int32_t)d;
        order_tokens[0] = 0;
        for (int64_t i = 0; i < D; ++i)
            order_tokens[(size_t)i + 1] = order_tokens[(size_t)i] + len_of(doc_order[(size_t)i]);
        // theta row slots: fixed capacity, so rows never move; laid out in the
        // order the documents are worked on, so that rows in use together are neighbours.
        // The buffer starts with 64 bytes of padding entries.
        slot_of.resize((size_t)D);
        h.slots_bytes = kSlotAlign;
        for (int64_t i = 0; i < D; ++i) {
            const int64_t d = doc_order[(size_t)i];
            if (h.slots_bytes / 16 > 0xffffffffull) return fail(MLDA_ENOTSUP, "theta rows need more than 64 GiB");
            slot_of[(size_t)d] = (uint32_t)(h.slots_bytes / 16);
            h.slots_bytes += slot_bytes_for(len_of(d), K, entry_bytes, max_count);
        }
        word_ptr.assign((size_t)V + 1, 0);
    } catch (const std::bad_alloc&) {
        return fail(MLDA_ENOMEM, "out of host memory");
    }

    // stable counting sort by word over parts of the length-sorted document sequence
    const int n_parts = (int)std::max<int64_t>(
        1, std::min<int64_t>({(int64_t)std::thread::hardware_concurrency(), 32, T / 65536 + 1}));
    std::vector<std::vector<int32_t>> part_hist(n_parts);
    std::vector<int> part_bad(n_parts, 0);
    // part p holds the documents doc_order[part_lo(p) .. part_lo(p+1)), about T/n_parts tokens
    auto part_lo = [&](int p) -> int64_t {
        if (p >= n_parts) return D;
        const int64_t want = T / n_parts * p;
        return std::lower_bound(order_tokens.begin(), order_tokens.end(), want) - order_tokens.begin();
    };
    const bool counted = parallel_chunks(n_parts, [&](int p) {
        auto& hist = part_hist[p];
        hist.assign((size_t)V, 0);
        for (int64_t i = part_lo(p); i < part_lo(p + 1); ++i) {
            const int64_t d = doc_order[(size_t)i];
            for (int64_t t = start_of(d); t < start_of(d) + len_of(d); ++t) {
                const int32_t w = word_ids[t];
                if (w < 0 || w >= V) { part_bad[p] = 1; return; }
                ++hist[w];
            }
        }
    });
    if (!counted) return fail(MLDA_ENOMEM, "out of host memory");
    for (int p = 0; p < n_parts; ++p)
        if (part_bad[p]) return fail(MLDA_EINVAL, "word id outside [0, V)");

    const int32_t tile = tile_tokens_for(K);
    size_t n_tiles = 0, n_segs = 0, n_split = 0;
    for (int32_t v = 0; v < V; ++v) {
        int32_t n = 0;
        for (int p = 0; p < n_parts; ++p) {
            const int32_t c = part_hist[p][v];
            part_hist[p][v] = n;            // becomes the part's offset inside the word
            n += c;
        }
        word_ptr[v + 1] = word_ptr[v] + n;
        n_tiles += (size_t)((n + tile - 1) / tile);
        n_segs += (size_t)((n + kPhiSegment - 1) / kPhiSegment);
        if (!accumulate && n > kPhiSegment) ++n_split;
    }
    h.n_tiles = (int32_t)n_tiles; h.n_segs = (int32_t)n_segs; h.n_split = (int32_t)n_split;
    h.L = chunk_layout(D, T, h.slots_bytes, n_tiles, n_segs, n_split, accumulate);

    h.release();
    h.pinned = pinned;
    if (pinned) {
        void* p = nullptr;
        if (hipHostMalloc(&p, std::max<size_t>(h.L.static_bytes, 1), hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            return fail(MLDA_ENOMEM, "out of pinned host memory");
        }
        h.arena = (unsigned char*)p;
    } else {
        h.arena = (unsigned char*)std::malloc(std::max<size_t>(h.L.static_bytes, 1));
        if (!h.arena) return fail(MLDA_ENOMEM, "out of host memory");
    }
    int32_t* tok_id = (int32_t*)(h.arena + h.L.tok_id);
    int32_t* doc_ptr32 = (int32_t*)(h.arena + h.L.doc_ptr);
    mlda::DocRec* doc_recs = (mlda::DocRec*)(h.arena + h.L.doc_order);
    uint2* row_rec = (uint2*)(h.arena + h.L.row_rec);
    mlda::Tile* tiles = (mlda::Tile*)(h.arena + h.L.tiles);
    mlda::Tile* segs = (mlda::Tile*)(h.arena + h.L.segs);
    int32_t* split_words = (int32_t*)(h.arena + h.L.split);

    // (the slot of every tile's middle document orders the tiles below)
    std::vector<uint32_t> tile_key;
    std::vector<int32_t> tile_base;
    try {
        tile_key.resize(n_tiles);
        tile_base.resize((size_t)V + 1);
    } catch (const std::bad_alloc&) {
        return fail(MLDA_ENOMEM, "out of host memory");
    }
    tile_base[0] = 0;
    for (int32_t v = 0; v < V; ++v)
        tile_base[v + 1] = tile_base[v] + (word_ptr[v + 1] - word_ptr[v] + tile - 1) / tile;
    const bool placed = parallel_chunks(n_parts, [&](int p) {
        auto& start = part_hist[p];
        for (int64_t i = part_lo(p); i < part_lo(p + 1); ++i) {
            const int64_t d = doc_order[(size_t)i];
            for (int64_t t = start_of(d); t < start_of(d) + len_of(d); ++t) {
                const int32_t w = word_ids[t];
                const int32_t in_word = start[w]++;
                tok_id[word_ptr[w] + in_word] = (int32_t)(tok_begin + t);   // the caller's token index keys the uniforms
                // the tile's middle token names the document whose slot is the tile's sort key
                const int32_t in_tile = in_word % tile;
                const int32_t tile_len = std::min(tile, word_ptr[w + 1] - word_ptr[w] - (in_word - in_tile));
                if (in_tile == tile_len / 2) tile_key[(size_t)(tile_base[w] + in_word / tile)] = slot_of[(size_t)d];
            }
        }
    });
    if (!placed) return fail(MLDA_ENOMEM, "out of host memory");
    part_hist.clear();

    for (int64_t d = 0; d < D; ++d) doc_ptr32[d] = (int32_t)start_of(d);
    doc_ptr32[D] = (int32_t)T;
    for (int64_t d = 0; d < D; ++d) row_rec[d] = make_uint2(slot_of[(size_t)d], 0u);
    for (int64_t i = 0; i < D; ++i) {
        const int64_t d = doc_order[(size_t)i];
        doc_recs[i] = mlda::DocRec{(int32_t)start_of(d), (int32_t)len_of(d), slot_of[(size_t)d], (int32_t)d};
    }
    // tiles and phi segments of one word each
    size_t it = 0, is = 0, ip = 0;
    for (int32_t v = 0; v < V; ++v) {
        const int32_t n = word_ptr[v + 1] - word_ptr[v];
        // a tile's `whole` carries its index until the tiles are sorted, then its word's wide row
        // of phi (mark_wide_tiles)
        for (int32_t b = 0; b < n; b += tile, ++it)
            tiles[it] = mlda::Tile{v, word_ptr[v] + b, std::min(tile, n - b), (int32_t)it};
        if (!accumulate && n > kPhiSegment) split_words[ip++] = v;
        for (int32_t b = 0; b < n; b += kPhiSegment)
            segs[is++] = mlda::Tile{v, word_ptr[v] + b, std::min(kPhiSegment, n - b),
                                    (!accumulate && n <= kPhiSegment) ? 1 : 0};
    }
    try {
        // Sampling tiles run in the order of their middle document (longest documents first;
        // slot offsets rise in that order), not word by word: tiles of different words that
        // are in flight together then walk the theta rows of the same documents, which are
        // fetched from HBM once instead of once per heavy word.  (The paper issues the tiles
        // of heavy words first, Section 6.1.2; here the long-row tiles come first, which also
        // keeps the tail short.)
        std::stable_sort(tiles, tiles + n_tiles, [&](const mlda::Tile& a, const mlda::Tile& b) {
            return tile_key[(size_t)a.whole] < tile_key[(size_t)b.whole];
        });
        std::stable_sort(segs, segs + n_segs,
                         [](const mlda::Tile& a, const mlda::Tile& b) { return a.count > b.count; });
        // tiles that hold a whole word of few tokens go last, to be taken in runs by one
        // workgroup each (their order among themselves stays)
        h.n_single = h.n_tiles;
        if (runs) {
            mlda::Tile* first_small = std::stable_partition(tiles, tiles + n_tiles, [&](const mlda::Tile& t) {
                const bool whole_word = word_ptr[t.word + 1] - word_ptr[t.word] == t.count;
                return !(whole_word && t.count <= mlda::kRunTileTokens);
            });
            h.n_single = (int32_t)(first_small - tiles);
            h.run_tokens = 0;
            for (const mlda::Tile* t = first_small; t < tiles + n_tiles; ++t) h.run_tokens += t->count;
        }
    } catch (const std::bad_alloc&) {
        return fail(MLDA_ENOMEM, "out of host memory");
    }
    return MLDA_OK;
}

// Chunk m of M covers the documents [chunk_first(m), chunk_first(m + 1)): about T / M tokens each.
int64_t chunk_first(const int64_t* doc_ptr, int64_t D, int32_t M, int32_t m) {
    if (m <= 0) return 0;
    if (m >= M) return D;
    const int64_t want = doc_ptr[D] / M * m;
    return std::lower_bound(doc_ptr, doc_ptr + D + 1, want) - doc_ptr;
}

}  // namespace

struct mlda_ctx {
    // ---- the corpus as a whole and the model
    int64_t D_all = 0, T_all = 0;
    int32_t V = 0, K = 0, Kpad = 0;
    double alpha = 0, beta = 0;
    uint64_t seed = 0;
    int32_t iter = 0;
    hipStream_t stream = nullptr;
    int n_cus = 0, lds_limit = 0;
    bool far_weights = false;           // p* of the sampler's tiles in device memory (large K)
    bool wide_slot_offsets = false;     // MLDA_WIDE_SLOT_OFFSETS: 64-bit unit addresses whatever the buffer's size
    float* far_pstar = nullptr;
    size_t sample_lds = 0;
    mlda::PhiView phi[2];                // [model_cur] is the current phi; two copies when streamed
    size_t phi_bytes = 0;                // bytes of one copy
    int32_t n_wide = 0;                  // words with an int32 row
    std::vector<int32_t> wide_row;       // [V] host copy of phi[].wide_row
    int32_t* n_k[2] = {nullptr, nullptr};
    int model_cur = 0;
    double *ll_partial = nullptr, *ll_scalars = nullptr;   // scalars: value, theta sum, document term
    double* lg_table = nullptr;          // lgG(c + alpha) - lgG(alpha), c < 1024, then lgG(alpha)
    double* lg_table_beta = nullptr;     // the same for beta
    unsigned long long* row_entries = nullptr;   // ring: [r % kEntryRing] written by rebuild r
    int64_t rebuilds = 0;                        // rebuilds launched so far
    int32_t last_step_iters = 0;
    bool has_state = false, ll_fresh = false;
    std::vector<hipEvent_t> events;     // 5 per timed iteration (streamed: kVisitEvents per timed visit)
    int32_t timed_iters = 0;            // iterations of the last step that carry events
    // streamed: what mlda_get_timing and mlda_get_sampler_bytes need of every timed chunk visit
    struct Visit {
        int32_t iter_row;               // row of the step's timed iterations
        int64_t T;
        int32_t n_tiles, n_wide_tiles;
        int64_t rebuild;                // number of the theta rebuild the visit's sampling read
        size_t event0;                  // first of its kVisitEvents events
    };
    std::vector<Visit> visit_log;

    // ---- the chunks (one: attached for good; several: attached in turn, Algorithm 1 WorkSchedule2)
    std::vector<HostChunk> chunks;
    bool streamed = false;
    unsigned char* slot_base[2] = {nullptr, nullptr};   // the workspace parts chunks are attached to
    uint16_t* z_host = nullptr;          // streamed: all assignments in the caller's order (pinned)
    hipStream_t copy_stream = nullptr;   // streamed: uploads run beside the kernels,
    hipStream_t down_stream = nullptr;   // and so do the downloads of new assignments
    hipEvent_t z_ready = nullptr;        // the attached chunk's assignments are in document order
    hipEvent_t slot_ready[2] = {nullptr, nullptr}, slot_free[2] = {nullptr, nullptr};
    std::vector<hipEvent_t> z_stored;    // per chunk: its assignments have reached z_host
    int64_t visits = 0;                  // chunk visits so far (picks the slot)

    // ---- the attached chunk
    const HostChunk* at = nullptr;
    int64_t D = 0, T = 0;
    uint32_t* tok_slot = nullptr;        // [T] slot of the theta row of each word-major token's document
    int32_t *tok_id = nullptr, *doc_map = nullptr, *doc_ptr = nullptr;
    uint2* doc_pairs = nullptr;          // streamed: {slot of the token's document, its topic}, document order
    mlda::DocRec* doc_order = nullptr;   // documents by falling length, as the theta rebuild walks them
    int32_t theta_grid = 0;
    bool tiny = false, wide_counters = false, short_docs = true;
    int32_t* split_words = nullptr;
    uint16_t* z[2] = {nullptr, nullptr}; // word-major assignments
    uint16_t* z_doc = nullptr;           // streamed: the same in document order (in doc_map's place)
    int cur = 0;
    uint2* row_rec = nullptr;
    unsigned char* slots = nullptr;
    size_t slots_bytes = 0;
    mlda::Tile* tiles = nullptr;         // sampling tiles
    mlda::Tile* segs = nullptr;          // phi rebuild segments
    int32_t n_tiles = 0, n_segs = 0, n_split = 0, n_wide_tiles = 0;
    int32_t n_single = 0;                // tiles taken one per workgroup; the rest in runs of run_tiles
    int32_t run_tiles = 1;
    int64_t run_tokens = 0;              // tokens of the tiles taken in runs

    int static_device = -1;              // >= 0: the workspace is that device's static array
};

// Workspace of contexts made by mlda_create_static: device memory that belongs to the library's
// code object, one copy per GPU, held until the process ends.  In host code the array's name
// is only a handle for hipGetSymbolAddress; kernels and copies take the address it returns.
static __device__ __align__(256) unsigned char scratch[MLDA_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};      // address of `scratch` on each device, once known
const mlda_ctx* g_scratch_user[kMaxDevices] = {};    // the live context that works in it, if any

// The current device's copy of `scratch`, claimed for `user`.  One context per device at a time.
int claim_scratch(const mlda_ctx* user, int* device, unsigned char** ptr) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(MLDA_ENOTSUP, "device index beyond the library's table");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_user[dev])
        return fail(MLDA_EINVAL, "this device's static workspace is in use by another context: "
                                 "destroy that context first");
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p) % kAlign != 0) return fail(MLDA_EHIP, "static workspace has no usable address");
        g_scratch_ptr[dev] = (unsigned char*)p;
    }
    g_scratch_user[dev] = user;
    *device = dev;
    *ptr = g_scratch_ptr[dev];
    return MLDA_OK;
}

void release_scratch(const mlda_ctx* user) {
    if (user->static_device < 0) return;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_user[user->static_device] == user) g_scratch_user[user->static_device] = nullptr;
}

int launch_check(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(MLDA_EHIP, std::string(what) + ": " + hipGetErrorString(e));
    return MLDA_OK;
}

int blocks_for(int64_t n, int per) { return (int)((n + per - 1) / per); }

// Point the context at chunk h in workspace part `base` (no data moves).
void point_at(mlda_ctx* c, const HostChunk& h, unsigned char* base) {
    c->at = &h;
    c->D = h.D; c->T = h.T;
    c->tiny = h.tiny;
    c->wide_counters = h.wide_counters;
    c->short_docs = h.short_docs;
    c->slots_bytes = h.slots_bytes;
    c->n_tiles = h.n_tiles; c->n_segs = h.n_segs; c->n_split = h.n_split;
    c->n_wide_tiles = h.n_wide_tiles;
    c->n_single = h.n_single;
    c->run_tokens = h.run_tokens;
    c->tok_slot = (uint32_t*)(base + h.L.tok_slot);
    c->tok_id = (int32_t*)(base + h.L.tok_id);
    c->doc_map = (int32_t*)(base + h.L.doc_map);
    c->doc_pairs = (uint2*)(base + h.L.doc_pairs);
    c->z_doc = (uint16_t*)(base + h.L.doc_map);   // a streamed chunk needs no map, see derive_chunk_arrays
    c->doc_ptr = (int32_t*)(base + h.L.doc_ptr);
    c->doc_order = (mlda::DocRec*)(base + h.L.doc_order);
    c->row_rec = (uint2*)(base + h.L.row_rec);
    c->tiles = (mlda::Tile*)(base + h.L.tiles);
    c->segs = (mlda::Tile*)(base + h.L.segs);
    c->split_words = (int32_t*)(base + h.L.split);
    c->z[0] = (uint16_t*)(base + h.L.z0);
    c->z[1] = (uint16_t*)(base + h.L.z1);
    c->slots = base + h.L.slots;
    c->cur = 0;
    const size_t theta_lds = mlda::theta_lds_bytes(c->K, h.wide_counters);
    // 16 one-wave workgroups per CU: enough to hide the gathers' latency; more of them
    // touch more lines of z at once than an XCD's L2 holds, and neighbours stop sharing
    const int per_cu = std::max(1, std::min(16, (int)(144 * 1024 / theta_lds)));
    c->theta_grid = (int32_t)std::min<int64_t>({h.D, (int64_t)c->n_cus * per_cu, (int64_t)kMaxThetaGrid});
}

// After the static part of a chunk has arrived: the index arrays that follow from it
// (document->token map, slot of every token's theta row), and what a lane of the sampler
// reads when it has no entries of its own: padding entries (count 0, topic K) in the 64 bytes
// before the first slot.  A streamed chunk arrives with its assignments in document order
// and hands them back so: its theta rebuilds read them directly and it needs no map (building
// one costs as much as a theta rebuild); the tokens' slots are then found by bisection.
void derive_chunk_arrays(mlda_ctx* c) {
    if (c->streamed) {
        // (the slots of a streamed chunk's tokens come with its assignments, see attach)
    } else if (c->T > 0) {
        hipLaunchKernelGGL(mlda::derive_doc_map_kernel, dim3(blocks_for(c->T, 256)), dim3(256), 0, c->stream,
                           c->tok_id, c->T, c->at->tok_begin, c->doc_map);
        const int grid = (int)std::min<int64_t>(c->D, (int64_t)c->n_cus * 32);
        hipLaunchKernelGGL(mlda::derive_tok_slot_kernel, dim3((unsigned)grid), dim3(mlda::kWave), 0, c->stream,
                           c->doc_order, c->D, c->doc_map, c->tok_slot);
        // from here on the map lists a document's tokens by rising place in z
        hipLaunchKernelGGL(mlda::sort_doc_map_kernel, dim3((unsigned)grid), dim3(mlda::kWave), 0, c->stream,
                           c->doc_order, c->D, c->doc_map);
    }
    const uint32_t pad = c->tiny ? (uint32_t)mlda::TinyRows::make(0, c->K) * 0x10001u
                                 : (uint32_t)mlda::PackedRows::make(0, c->K);
    static_assert(kSlotAlign >= (mlda::kKeptUnits + 1) * 16, "the padding units lie before the first slot");
    hipLaunchKernelGGL(mlda::fill_i32_kernel, dim3(1), dim3(256), 0, c->stream, (int32_t*)c->slots,
                       (int64_t)(kSlotAlign / 4), (int32_t)pad);
}

// Streamed: bring chunk m into the slot of this visit.  The static part (and with_z: the
// chunk's assignments, caller's order, into z_doc) is copied on the copy stream, so that it
// overlaps the kernels of the chunk before; the context's stream then waits for it and, with_z,
// also puts the assignments in word-major order into z[0].
int attach(mlda_ctx* c, int32_t m, bool with_z, hipEvent_t* ev = nullptr) {
    const HostChunk& h = c->chunks[(size_t)m];
    const int s = (int)(c->visits % 2);
    c->visits += 1;
    point_at(c, h, c->slot_base[s]);
    // the slot's previous user must be done, and this chunk's last assignments stored
    HIP_TRY(hipStreamWaitEvent(c->copy_stream, c->slot_free[s], 0));
    if (h.L.static_bytes > 0)
        HIP_TRY(hipMemcpyAsync(c->slot_base[s], h.arena, h.L.static_bytes, hipMemcpyHostToDevice,
                               c->copy_stream));
    if (with_z && h.T > 0) {
        HIP_TRY(hipStreamWaitEvent(c->copy_stream, c->z_stored[(size_t)m], 0));
        HIP_TRY(hipMemcpyAsync(c->z_doc, c->z_host + h.tok_begin, (size_t)h.T * 2, hipMemcpyHostToDevice,
                               c->copy_stream));
    }
    HIP_TRY(hipEventRecord(c->slot_ready[s], c->copy_stream));
    HIP_TRY(hipStreamWaitEvent(c->stream, c->slot_ready[s], 0));
    if (ev) HIP_TRY(hipEventRecord(ev[0], c->stream));
    derive_chunk_arrays(c);
    if (with_z && h.T > 0) {
        // every token's topic is paired with the slot of its document's theta row where both
        // are contiguous, and the pairs are then brought to word-major order in one gather
        const int grid = (int)std::min<int64_t>(h.D, (int64_t)c->n_cus * 32);
        hipLaunchKernelGGL(mlda::pair_topics_with_slots_kernel, dim3((unsigned)grid), dim3(mlda::kWave), 0,
                           c->stream, c->doc_order, h.D, c->z_doc, c->doc_pairs);
        hipLaunchKernelGGL(mlda::pairs_to_word_major_kernel, dim3(blocks_for(h.T, 256)), dim3(256), 0,
                           c->stream, c->doc_pairs, c->tok_id, c->z[0], c->tok_slot, h.T, h.tok_begin);
    }
    if (ev) HIP_TRY(hipEventRecord(ev[1], c->stream));
    return launch_check("attaching a chunk");
}

// Streamed: new word-major assignments of the attached chunk, put in document order too.
int to_document_order(mlda_ctx* c, const uint16_t* z_word) {
    if (c->T > 0)
        hipLaunchKernelGGL(mlda::to_doc_major_scatter_kernel, dim3(blocks_for(c->T, 256)), dim3(256), 0,
                           c->stream, z_word, c->tok_id, c->z_doc, c->T, c->at->tok_begin);
    return launch_check("to_doc_major_scatter_kernel");
}

// Streamed: the attached chunk's assignments (z_doc) go back to the host if `store`, and the
// chunk's slot is free again once everything queued so far is done.
int store_z_and_release(mlda_ctx* c, int32_t m, bool store) {
    const HostChunk& h = c->chunks[(size_t)m];
    const int s = (int)((c->visits - 1) % 2);
    if (store && h.T > 0) {
        // the download runs on its own stream, beside the next chunk's kernels and upload
        HIP_TRY(hipEventRecord(c->z_ready, c->stream));
        HIP_TRY(hipStreamWaitEvent(c->down_stream, c->z_ready, 0));
        HIP_TRY(hipMemcpyAsync(c->z_host + h.tok_begin, c->z_doc, (size_t)h.T * 2, hipMemcpyDeviceToHost,
                               c->down_stream));
        HIP_TRY(hipEventRecord(c->z_stored[(size_t)m], c->down_stream));
        HIP_TRY(hipEventRecord(c->slot_free[s], c->down_stream));
    } else {
        HIP_TRY(hipEventRecord(c->slot_free[s], c->stream));
    }
    return MLDA_OK;
}

// phi (into n_wk[which]) from the attached chunk's assignments z (word-major).  One chunk:
// rows are stored and n_k follows; several: the chunk's counts are added to a phi that was
// zeroed before the first chunk, and n_k is formed after the last (finish_model).
int rebuild_phi(mlda_ctx* c, const uint16_t* z, int which) {
    using namespace mlda;
    // one counter per topic in LDS; K beyond kHistTopics is counted range by range
    const int32_t span = std::min<int32_t>(c->K, kHistTopics);
    const size_t hist_bytes = (size_t)span * 4;
    const bool ranges = c->K > kHistTopics;
    if (!c->streamed) {
        if (c->n_split > 0) {
            dim3 grid((unsigned)c->n_split, (unsigned)blocks_for(c->K, 256));
            hipLaunchKernelGGL(zero_rows_kernel, grid, dim3(256), 0, c->stream, c->split_words,
                               c->phi[which], c->K);
        }
        hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks_for(c->K, 256)), dim3(256), 0, c->stream,
                           c->n_k[which], (int64_t)c->K, 0);
    }
    if (c->n_tiles > 0) {
        if (!ranges)
            hipLaunchKernelGGL(phi_tile_kernel<false>, dim3((unsigned)c->n_segs), dim3(256), hist_bytes, c->stream,
                               c->segs, z, c->phi[which], c->K, 0, c->K);
        else
            for (int32_t k_lo = 0; k_lo < c->K; k_lo += span)
                hipLaunchKernelGGL(phi_tile_kernel<true>, dim3((unsigned)c->n_segs), dim3(256), hist_bytes,
                                   c->stream, c->segs, z, c->phi[which], c->K, k_lo, std::min(span, c->K - k_lo));
        if (c->streamed) {
            // n_k after the last chunk
        } else if ((int64_t)c->V * c->K * 2 < c->T) {
            // n_k as column sums of the fresh n_wk: fewer bytes than z and no LDS atomics
            const int words_per_slice = 64;
            dim3 grid((unsigned)blocks_for(c->K, 256), (unsigned)blocks_for(c->V, words_per_slice));
            hipLaunchKernelGGL(topic_totals_from_rows_kernel, grid, dim3(256), 0, c->stream,
                               c->phi[which], c->V, c->n_wide, c->K, words_per_slice, c->n_k[which]);
        } else {
            const int grid = (int)std::min<int64_t>((c->T + 4095) / 4096, (int64_t)c->n_cus * 8);
            if (!ranges)
                hipLaunchKernelGGL(topic_totals_kernel<false>, dim3((unsigned)grid), dim3(256), hist_bytes,
                                   c->stream, z, c->T, c->n_k[which], c->K, 0, c->K);
            else
                for (int32_t k_lo = 0; k_lo < c->K; k_lo += span)
                    hipLaunchKernelGGL(topic_totals_kernel<true>, dim3((unsigned)grid), dim3(256), hist_bytes,
                                       c->stream, z, c->T, c->n_k[which], c->K, k_lo, std::min(span, c->K - k_lo));
        }
    }
    return launch_check("phi rebuild kernels");
}

// Streamed: phi[which] starts at zero before the first chunk adds to it ...
int begin_model(mlda_ctx* c, int which) {
    const int64_t dwords = (int64_t)(c->phi_bytes / 4);
    hipLaunchKernelGGL(mlda::fill_i32_kernel, dim3(blocks_for(dwords, 256)), dim3(256), 0, c->stream,
                       (int32_t*)c->phi[which].narrow, dwords, 0);
    return launch_check("fill_i32_kernel");
}

// ... and n_k[which] is its column sums after the last.
int finish_model(mlda_ctx* c, int which) {
    hipLaunchKernelGGL(mlda::fill_i32_kernel, dim3(blocks_for(c->K, 256)), dim3(256), 0, c->stream,
                       c->n_k[which], (int64_t)c->K, 0);
    const int words_per_slice = 64;
    dim3 grid((unsigned)blocks_for(c->K, 256), (unsigned)blocks_for(c->V, words_per_slice));
    hipLaunchKernelGGL(mlda::topic_totals_from_rows_kernel, grid, dim3(256), 0, c->stream, c->phi[which],
                       c->V, c->n_wide, c->K, words_per_slice, c->n_k[which]);
    return launch_check("topic totals");
}

// theta rows of the attached chunk from its assignments: z word-major, reached through the
// document->token map; streamed: z = z_doc, read directly.  Leaves the rows' part of the
// log-likelihood as one partial per workgroup in ll_partial[2 kLoglikBlocks ..].
int rebuild_theta(mlda_ctx* c, const uint16_t* z) {
    using namespace mlda;
    const int32_t* doc_map = c->streamed ? nullptr : c->doc_map;
    if (c->D > 0) {
        const size_t theta_lds = theta_lds_bytes(c->K, c->wide_counters);
        unsigned long long* entries = c->row_entries + (c->rebuilds % kEntryRing);
        hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, c->stream, entries);
        // two documents per wave where a half-wave suits them: few topics, short documents
        const bool pairs = c->K <= kPairMaxK && !c->wide_counters && c->T <= 160 * c->D;
        const void* kernel =
            pairs ? (c->tiny ? (const void*)theta_rows_pair_kernel<TinyRows> : (const void*)theta_rows_pair_kernel<PackedRows>)
                  : theta_kernel_for(c->tiny, c->wide_counters);
        const size_t lds = pairs ? theta_pair_lds_bytes(c->K) : theta_lds;
        const DocRec* docs = c->doc_order;
        uint2* row_rec = c->row_rec;
        unsigned char* slots = c->slots;
        int64_t D = c->D, T = c->T;
        int32_t K = c->K;
        double alpha = c->alpha;
        const double* lg_table = c->lg_table;
        double* ll_partial = c->ll_partial + 2 * kLoglikBlocks;
        void* args[] = {&docs, &doc_map, &z, &row_rec, &slots, &D, &T, &K, &alpha, &lg_table, &entries, &ll_partial};
        HIP_TRY(hipLaunchKernel(kernel, dim3((unsigned)c->theta_grid), dim3(kWave), args, lds, c->stream));
    }
    c->rebuilds += 1;
    return launch_check("theta rebuild kernel");
}

int launch_sampler(mlda_ctx* c, const uint16_t* z_cur, uint16_t* z_next) {
    if (c->n_tiles == 0) return MLDA_OK;
    mlda::SampleArgs a;
    a.tiles = c->tiles;
    a.tok_slot = c->tok_slot;
    a.tok_id = c->tok_id;
    a.z_cur = z_cur;
    a.z_next = z_next;
    a.slots = c->slots;
    a.phi = c->phi[c->model_cur];
    a.n_k = c->n_k[c->model_cur];
    a.K = c->K;
    a.Kpad = c->Kpad;
    a.alpha = c->alpha;
    a.beta = c->beta;
    a.beta_V = c->beta * (double)c->V;
    a.seed = c->seed;
    a.iter = (uint32_t)(c->iter + 1);
    a.n_tiles = c->n_tiles;
    a.n_single = c->run_tiles > 1 ? c->n_single : c->n_tiles;
    a.run_tiles = c->run_tiles;
    a.far_pstar = c->far_pstar;
    const int waves = sample_waves_for(c->K);
    const int32_t grid = c->far_weights ? std::min<int32_t>(a.n_tiles, kFarStrips)
                                        : a.n_single + (a.n_tiles - a.n_single + a.run_tiles - 1) / a.run_tiles;
    void* kernel_args[] = {&a};
    HIP_TRY(hipLaunchKernel(sample_kernel_for(c->K, c->short_docs, slots_near(c->slots_bytes) && !c->wide_slot_offsets),
                            dim3((unsigned)grid),
                            dim3((unsigned)(waves * mlda::kWave)), kernel_args, c->sample_lds, c->stream));
    return launch_check("sample_kernel");
}

// Log-likelihood of the current state, one chunk: word side, document term, theta partials
// left by the last rebuild_theta.
int launch_loglik(mlda_ctx* c) {
    using namespace mlda;
    hipLaunchKernelGGL(loglik_word_side_kernel, dim3(kLoglikBlocks), dim3(256), 0, c->stream,
                       c->phi[c->model_cur], (int64_t)c->V * c->K, (int64_t)c->n_wide * c->K,
                       c->n_k[c->model_cur], c->K, c->beta,
                       (double)c->V * c->beta, c->lg_table_beta, c->ll_partial);
    hipLaunchKernelGGL(loglik_doc_term_kernel, dim3(kLoglikBlocks), dim3(256), 0, c->stream, c->doc_ptr,
                       c->D, (double)c->K * c->alpha, c->ll_partial + kLoglikBlocks);
    hipLaunchKernelGGL(loglik_final_kernel, dim3(1), dim3(256), 0, c->stream, c->ll_partial,
                       2 * kLoglikBlocks + c->theta_grid, (const double*)nullptr, 0, c->ll_scalars);
    c->ll_fresh = true;
    return launch_check("log-likelihood kernels");
}

// Streamed: the theta partials of the chunk just rebuilt are added to the running sum ...
int add_theta_loglik(mlda_ctx* c, bool first) {
    hipLaunchKernelGGL(mlda::loglik_final_kernel, dim3(1), dim3(256), 0, c->stream,
                       c->ll_partial + 2 * kLoglikBlocks, c->D > 0 ? c->theta_grid : 0,
                       (const double*)nullptr, first ? 0 : 1, c->ll_scalars + 1);
    return launch_check("loglik_final_kernel");
}

// ... and the value is the word side plus that sum plus the documents' term (a constant of
// the corpus, scalars[2]).
int finish_loglik_streamed(mlda_ctx* c) {
    using namespace mlda;
    hipLaunchKernelGGL(loglik_word_side_kernel, dim3(kLoglikBlocks), dim3(256), 0, c->stream,
                       c->phi[c->model_cur], (int64_t)c->V * c->K, (int64_t)c->n_wide * c->K,
                       c->n_k[c->model_cur], c->K, c->beta,
                       (double)c->V * c->beta, c->lg_table_beta, c->ll_partial);
    hipLaunchKernelGGL(loglik_final_kernel, dim3(1), dim3(256), 0, c->stream, c->ll_partial, kLoglikBlocks,
                       (const double*)(c->ll_scalars + 1), 0, c->ll_scalars);
    hipLaunchKernelGGL(loglik_final_kernel, dim3(1), dim3(256), 0, c->stream, c->ll_partial, 0,
                       (const double*)(c->ll_scalars + 2), 1, c->ll_scalars);
    c->ll_fresh = true;
    return launch_check("log-likelihood kernels");
}

int need_state(const mlda_ctx* c) {
    if (!c) return fail(MLDA_EINVAL, "null context");
    if (!c->has_state)
        return fail(MLDA_EINVAL, "no topic assignments yet: call mlda_init_random or mlda_set_assignments");
    return MLDA_OK;
}

int check_corpus(const int64_t* doc_ptr, const int32_t* word_ids, bool need_words, int64_t D, int32_t V,
                 int32_t K, double alpha, double beta) {
    if (!doc_ptr) return fail(MLDA_EINVAL, "doc_ptr is null");
    if (D < 0 || V < 1) return fail(MLDA_EINVAL, "need D >= 0 and V >= 1");
    if (K < 1 || K > 65535) return fail(MLDA_EINVAL, "K must be in [1, 65535] (16-bit topic indices)");
    if (!(alpha > 0.0) || !(beta > 0.0) || !std::isfinite(alpha) || !std::isfinite(beta))
        return fail(MLDA_EINVAL, "alpha and beta must be positive and finite");
    if (doc_ptr[0] != 0) return fail(MLDA_EINVAL, "doc_ptr[0] must be 0");
    for (int64_t d = 0; d < D; ++d)
        if (doc_ptr[d + 1] < doc_ptr[d]) return fail(MLDA_EINVAL, "doc_ptr must be non-decreasing");
    if (doc_ptr[D] >= ((int64_t)1 << 31)) return fail(MLDA_EINVAL, "2^31 or more tokens");
    if (need_words && doc_ptr[D] > 0 && !word_ids) return fail(MLDA_EINVAL, "word_ids is null");
    return MLDA_OK;
}

int check_workspace(void* dev_workspace, size_t have, size_t need) {
    if (!dev_workspace) return fail(MLDA_EINVAL, "dev_workspace is null");
    if (((uintptr_t)dev_workspace) % kAlign != 0)
        return fail(MLDA_EINVAL, "dev_workspace must be 256-byte aligned");
    if (have < need)
        return fail(MLDA_ENOMEM, "workspace has " + std::to_string(have) + " bytes, need " +
                                     std::to_string(need));
    return MLDA_OK;
}

int check_device_pointer(void* dev_workspace) {
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, dev_workspace);
    if (e != hipSuccess || attr.type != hipMemoryTypeDevice) {
        (void)hipGetLastError();
        return fail(MLDA_EINVAL, "dev_workspace is not device memory");
    }
    return MLDA_OK;
}

size_t streamed_workspace_bound(const int64_t* doc_ptr, int64_t D, int32_t V, int32_t K, int32_t M) {
    size_t chunk = 0;
    for (int32_t m = 0; m < M; ++m) {
        const int64_t a = chunk_first(doc_ptr, D, M, m), b = chunk_first(doc_ptr, D, M, m + 1);
        chunk = std::max(chunk, chunk_layout_bound(b - a, doc_ptr[b] - doc_ptr[a], V, K, true).total);
    }
    return model_layout(V, K, doc_ptr[D], true).total + 2 * chunk;
}

// Everything mlda_create and mlda_create_streamed share: device limits, the model's buffers
// and tables.  `chunks` are prepared; `base` is the workspace.
int finish_create(mlda_ctx* c, unsigned char* base, const ModelLayout& ML) {
    for (int i = 0; i < 2; ++i) {
        c->phi[i].narrow = (uint16_t*)(base + ML.phi[i]);
        c->phi[i].wide = (int32_t*)(base + ML.phi[i] + ML.phi_wide);
        c->phi[i].wide_row = (const int32_t*)(base + ML.wide_row);
    }
    c->phi_bytes = ML.phi_bytes;
    HIP_TRY(hipMemcpyAsync(base + ML.wide_row, c->wide_row.data(), (size_t)c->V * 4, hipMemcpyHostToDevice,
                           c->stream));
    c->n_k[0] = (int32_t*)(base + ML.n_k[0]);
    c->n_k[1] = (int32_t*)(base + ML.n_k[1]);
    c->ll_partial = (double*)(base + ML.ll_partial);
    c->ll_scalars = (double*)(base + ML.ll_scalars);
    c->lg_table = (double*)(base + ML.lg_table);
    c->lg_table_beta = c->lg_table + (mlda::kLgTable + 1);
    c->row_entries = (unsigned long long*)(base + ML.row_entries);
    c->far_pstar = (float*)(base + ML.far_pstar);

    hipLaunchKernelGGL(mlda::lg_table_kernel, dim3(blocks_for(mlda::kLgTable + 1, 256)), dim3(256), 0,
                       c->stream, c->lg_table, c->alpha);
    hipLaunchKernelGGL(mlda::lg_table_kernel, dim3(blocks_for(mlda::kLgTable + 1, 256)), dim3(256), 0,
                       c->stream, c->lg_table_beta, c->beta);
    // rows of words without tokens are never written again: start phi at zero
    const int64_t dwords = (int64_t)(c->phi_bytes / 4);
    hipLaunchKernelGGL(mlda::fill_i32_kernel, dim3(blocks_for(dwords, 256)), dim3(256), 0, c->stream,
                       (int32_t*)c->phi[0].narrow, dwords, 0);
    RC_TRY(launch_check("model set-up kernels"));
    if (c->sample_lds > 48 * 1024)
        for (bool short_docs : {false, true})
            for (bool near : {false, true})
                // (the attribute belongs to the kernel, not to this context: contexts of different
                // needs may live side by side, so it is raised to what the device allows)
                HIP_TRY(hipFuncSetAttribute(sample_kernel_for(c->K, short_docs, near),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, c->lds_limit));
    if ((size_t)c->K * 4 > 48 * 1024) {
        const int hist_bytes = std::min<int32_t>(c->K, kHistTopics) * 4;
        for (const void* kernel : {(const void*)mlda::phi_tile_kernel<false>, (const void*)mlda::phi_tile_kernel<true>,
                                   (const void*)mlda::topic_totals_kernel<false>,
                                   (const void*)mlda::topic_totals_kernel<true>})
            HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, hist_bytes));
    }
    for (bool wide : {false, true})
        if (mlda::theta_lds_bytes(c->K, wide) > 48 * 1024 &&
            mlda::theta_lds_bytes(c->K, wide) <= (size_t)c->lds_limit)      // (else see check_theta_lds)
            HIP_TRY(hipFuncSetAttribute(theta_kernel_for(tiny_rows_for(c->K), wide),
                                        hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)mlda::theta_lds_bytes(c->K, wide)));
    return MLDA_OK;
}

// The theta rebuild keeps counters per topic in LDS: 16-bit ones for all topics, or, once a
// document of the chunk has 2^16 tokens or more, 32-bit ones for up to 32,768 topics at a time.
// On a device that allows a workgroup the 160 KB this library is written for they always fit.
int check_theta_lds(const mlda_ctx* c, const HostChunk& h) {
    const size_t need = mlda::theta_lds_bytes(c->K, h.wide_counters);
    if (need > (size_t)c->lds_limit)
        return fail(MLDA_ENOTSUP, "K = " + std::to_string(c->K) + " needs " + std::to_string(need) +
                                      " bytes of LDS per workgroup for the theta rebuild, the device allows " +
                                      std::to_string(c->lds_limit));
    return MLDA_OK;
}

// Which words get an int32 row of phi: those with 2^16 tokens or more in the whole corpus.
int find_wide_rows(mlda_ctx* c, const int32_t* word_ids) {
    try {
        const int n_parts = (int)std::max<int64_t>(1, std::min<int64_t>(8, c->T_all >> 22));
        std::vector<std::vector<int32_t>> hist((size_t)n_parts);
        const int64_t per = (c->T_all + n_parts - 1) / n_parts;
        const bool ok = parallel_chunks(n_parts, [&](int p) {
            hist[(size_t)p].assign((size_t)c->V, 0);
            auto& h = hist[(size_t)p];
            const int32_t V = c->V;
            for (int64_t t = per * p; t < std::min(c->T_all, per * (p + 1)); ++t) {
                const int32_t w = word_ids[t];
                if (w >= 0 && w < V) h[(size_t)w] += 1;      // (ids out of range are reported later)
            }
        });
        if (!ok) return fail(MLDA_ENOMEM, "out of host memory");
        c->wide_row.assign((size_t)c->V, -1);
        c->n_wide = 0;
        for (int32_t v = 0; v < c->V; ++v) {
            int64_t n = 0;
            for (int p = 0; p < n_parts; ++p) n += hist[(size_t)p][(size_t)v];
            if (n >= mlda::kNarrowWordLimit) c->wide_row[(size_t)v] = c->n_wide++;
        }
    } catch (const std::bad_alloc&) {
        return fail(MLDA_ENOMEM, "out of host memory");
    }
    return MLDA_OK;
}

// Every sampling tile carries its word's row among the wide rows of phi (or -1).
void mark_wide_tiles(const mlda_ctx* c, HostChunk& h) {
    mlda::Tile* tiles = (mlda::Tile*)(h.arena + h.L.tiles);
    h.n_wide_tiles = 0;
    for (int32_t i = 0; i < h.n_tiles; ++i) {
        tiles[i].whole = c->wide_row[(size_t)tiles[i].word];
        if (tiles[i].whole >= 0) h.n_wide_tiles += 1;
    }
}

int device_limits(mlda_ctx* c) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&c->n_cus, hipDeviceAttributeMultiprocessorCount, dev));
    HIP_TRY(hipDeviceGetAttribute(&c->lds_limit, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
    c->Kpad = kpad_for(c->K);
    c->far_weights = far_weights_for(c->K);
    // (a switch for tests: the 64-bit form is otherwise only reached by theta slots beyond 4 GiB)
    const char* wide = std::getenv("MLDA_WIDE_SLOT_OFFSETS");
    c->wide_slot_offsets = wide && wide[0] != '\0' && wide[0] != '0';
    c->sample_lds = c->far_weights ? mlda::sample_far_lds_bytes(c->Kpad, sample_waves_for(c->K))
                                   : mlda::sample_lds_bytes(c->Kpad, sample_waves_for(c->K));
    if (c->sample_lds > (size_t)c->lds_limit)
        return fail(MLDA_ENOTSUP, "K = " + std::to_string(c->K) + " needs " + std::to_string(c->sample_lds) +
                                      " bytes of LDS per workgroup, the device allows " +
                                      std::to_string(c->lds_limit));
    // Large K, corpus resident (so that phi holds exactly the attached tokens): the many words
    // of few tokens are sampled in runs, one workgroup turning p* of one word into p* of the
    // next.  That takes a little more LDS; not if it would cost the CU its second workgroup.
    c->run_tiles = 1;
    const size_t with_runs = c->sample_lds + mlda::sample_run_lds_bytes(c->Kpad, sample_waves_for(c->K));
    const size_t cu_lds = 160 * 1024;
    if (sample_waves_for(c->K) == 12 && !c->far_weights && !c->streamed && with_runs <= (size_t)c->lds_limit &&
        (2 * with_runs <= cu_lds || 2 * c->sample_lds > cu_lds)) {
        c->sample_lds = with_runs;
        c->run_tiles = kRunTiles;
    }
    return MLDA_OK;
}

void destroy(mlda_ctx* c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    for (hipStream_t extra : {c->copy_stream, c->down_stream})
        if (extra) {
            (void)hipStreamSynchronize(extra);
            (void)hipStreamDestroy(extra);
        }
    if (c->z_ready) (void)hipEventDestroy(c->z_ready);
    for (hipEvent_t ev : c->events) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : c->z_stored) (void)hipEventDestroy(ev);
    for (int s = 0; s < 2; ++s) {
        if (c->slot_ready[s]) (void)hipEventDestroy(c->slot_ready[s]);
        if (c->slot_free[s]) (void)hipEventDestroy(c->slot_free[s]);
    }
    if (c->z_host) (void)hipHostFree(c->z_host);
    release_scratch(c);
    delete c;
}

// Rows of theta of the attached chunk, unpacked into the caller's CSR arrays (documents
// h.d_begin ..; row_ptr already holds the row starts).
int fetch_rows(mlda_ctx* c, std::vector<uint2>& rec, std::vector<unsigned char>& slots) {
    try {
        rec.resize((size_t)c->D);
        slots.resize(c->slots_bytes);
    } catch (const std::bad_alloc&) {
        return fail(MLDA_ENOMEM, "out of host memory");
    }
    if (c->D > 0)
        HIP_TRY(hipMemcpyAsync(rec.data(), c->row_rec, (size_t)c->D * 8, hipMemcpyDeviceToHost, c->stream));
    if (c->slots_bytes > 0)
        HIP_TRY(hipMemcpyAsync(slots.data(), c->slots, c->slots_bytes, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return MLDA_OK;
}

int fetch_row_rec(mlda_ctx* c, std::vector<uint2>& rec) {
    try { rec.resize((size_t)c->D); } catch (const std::bad_alloc&) {
        return fail(MLDA_ENOMEM, "out of host memory");
    }
    if (c->D > 0)
        HIP_TRY(hipMemcpyAsync(rec.data(), c->row_rec, (size_t)c->D * 8, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return MLDA_OK;
}

// rec[d].y = distinct topics of row d (the length of its CSR row); the slot's header holds the
// number of entries, of which several in a row may share a topic (a count spread over them).
template <class Layout>
void unpack_rows_as(const mlda_ctx* c, const std::vector<uint2>& rec, const std::vector<unsigned char>& slots,
                    const int64_t* row_ptr, uint16_t* topics, int32_t* counts) {
    typedef typename Layout::Entry Entry;
    for (int64_t d = 0; d < c->D; ++d) {
        if (rec[(size_t)d].y == 0) continue;
        const unsigned char* head = slots.data() + (size_t)rec[(size_t)d].x * 16;
        uint32_t n_entries;
        std::memcpy(&n_entries, head, 4);
        const Entry* ent = reinterpret_cast<const Entry*>(head + mlda::kRowHeader);
        int64_t at = row_ptr[d] - 1;
        int last_topic = -1;
        for (uint32_t j = 0; j < n_entries; ++j) {
            const int topic = Layout::entry_topic(ent[j]), count = Layout::entry_count(ent[j]);
            if (topic != last_topic) {
                ++at;
                topics[at] = (uint16_t)topic;
                counts[at] = 0;
                last_topic = topic;
            }
            counts[at] += count;
        }
    }
}

void unpack_rows(const mlda_ctx* c, const std::vector<uint2>& rec, const std::vector<unsigned char>& slots,
                 const int64_t* row_ptr, uint16_t* topics, int32_t* counts) {
    if (c->tiny) unpack_rows_as<mlda::TinyRows>(c, rec, slots, row_ptr, topics, counts);
    else unpack_rows_as<mlda::PackedRows>(c, rec, slots, row_ptr, topics, counts);
}

// Streamed: phi and n_k of the assignments in z_host (after init or set_assignments);
// `init`: the assignments are drawn on the device first and stored.
int rebuild_model_streamed(mlda_ctx* c, bool init) {
    RC_TRY(begin_model(c, c->model_cur));
    for (int32_t m = 0; m < (int32_t)c->chunks.size(); ++m) {
        if (c->chunks[(size_t)m].D == 0) continue;
        RC_TRY(attach(c, m, !init));
        if (init && c->T > 0)
            hipLaunchKernelGGL(mlda::init_topics_kernel, dim3(blocks_for(c->T, 256)), dim3(256), 0, c->stream,
                               c->tok_id, c->z[0], c->T, c->K, c->seed);
        RC_TRY(rebuild_phi(c, c->z[0], c->model_cur));
        if (init) RC_TRY(to_document_order(c, c->z[0]));
        RC_TRY(store_z_and_release(c, m, init));
    }
    return finish_model(c, c->model_cur);
}

// Streamed: the theta rows of every chunk are rebuilt in turn from z_host; `visit` sees each
// attached chunk with its rows in place.  Also leaves the log-likelihood's theta sum.
template <class F>
int for_each_chunk_rows(mlda_ctx* c, F&& visit) {
    bool first = true;
    for (int32_t m = 0; m < (int32_t)c->chunks.size(); ++m) {
        if (c->chunks[(size_t)m].D == 0) continue;
        RC_TRY(attach(c, m, true));
        RC_TRY(rebuild_theta(c, c->z_doc));
        RC_TRY(add_theta_loglik(c, first));
        first = false;
        RC_TRY(visit(c->chunks[(size_t)m]));
        RC_TRY(store_z_and_release(c, m, false));
    }
    if (first) {            // no documents at all: the sum is empty
        hipLaunchKernelGGL(mlda::loglik_final_kernel, dim3(1), dim3(256), 0, c->stream, c->ll_partial, 0,
                           (const double*)nullptr, 0, c->ll_scalars + 1);
        RC_TRY(launch_check("loglik_final_kernel"));
    }
    return MLDA_OK;
}

}  // namespace

extern "C" {

const char* mlda_strerror(int code) {
    switch (code) {
        case MLDA_OK: return "ok";
        case MLDA_EINVAL: return "invalid argument";
        case MLDA_ENOMEM: return "workspace too small or out of host memory";
        case MLDA_EHIP: return "HIP call failed";
        case MLDA_ENOTSUP: return "beyond what the device or the library supports";
        default: return "unknown error";
    }
}

const char* mlda_last_error(void) { return g_last_error.c_str(); }

int mlda_workspace_bytes(int64_t D, int64_t T, int32_t V, int32_t K, size_t* bytes) {
    if (!bytes) return fail(MLDA_EINVAL, "bytes is null");
    if (D < 0 || T < 0 || V < 1 || K < 1 || K > 65535 || T >= ((int64_t)1 << 31))
        return fail(MLDA_EINVAL, "need D >= 0, 0 <= T < 2^31, V >= 1, 1 <= K <= 65535");
    *bytes = model_layout(V, K, T, false).total + chunk_layout_bound(D, T, V, K, false).total;
    return MLDA_OK;
}

int mlda_workspace_bytes_streamed(const int64_t* doc_ptr, int64_t D, int32_t V, int32_t K,
                                  int32_t n_chunks, size_t* bytes) {
    if (!bytes) return fail(MLDA_EINVAL, "bytes is null");
    RC_TRY(check_corpus(doc_ptr, nullptr, false, D, V, K, 1.0, 1.0));
    if (n_chunks < 1) return fail(MLDA_EINVAL, "n_chunks must be >= 1");
    *bytes = streamed_workspace_bound(doc_ptr, D, V, K, n_chunks);
    return MLDA_OK;
}

// mlda_create and mlda_create_static: the corpus resident in one workspace.  With
// `in_static` the workspace is the current device's static array, claimed here.
static int create_resident(mlda_ctx** out, const int64_t* doc_ptr, const int32_t* word_ids, int64_t D,
                           int32_t V, int32_t K, double alpha, double beta, uint64_t seed,
                           void* dev_workspace, size_t workspace_bytes, void* hip_stream, bool in_static) {
    if (!out) return fail(MLDA_EINVAL, "out is null");
    *out = nullptr;
    RC_TRY(check_corpus(doc_ptr, word_ids, true, D, V, K, alpha, beta));
    const int64_t T = doc_ptr[D];
    size_t need_bound = 0;
    if (mlda_workspace_bytes(D, T, V, K, &need_bound) != MLDA_OK) return MLDA_EINVAL;
    if (in_static) {
        if (need_bound > (size_t)MLDA_STATIC_WORKSPACE_BYTES)
            return fail(MLDA_ENOMEM, "this corpus needs a workspace of " + std::to_string(need_bound) +
                                         " bytes, the static one holds " +
                                         std::to_string((size_t)MLDA_STATIC_WORKSPACE_BYTES) +
                                         ": use mlda_create with a workspace of the caller's");
    } else {
        RC_TRY(check_workspace(dev_workspace, workspace_bytes, need_bound));
        RC_TRY(check_device_pointer(dev_workspace));
    }
    mlda_ctx* c = new (std::nothrow) mlda_ctx();
    if (!c) return fail(MLDA_ENOMEM, "out of host memory");
    if (in_static) {
        unsigned char* ptr = nullptr;
        const int rc_claim = claim_scratch(c, &c->static_device, &ptr);
        if (rc_claim != MLDA_OK) { delete c; return rc_claim; }
        dev_workspace = ptr;
        workspace_bytes = (size_t)MLDA_STATIC_WORKSPACE_BYTES;
    }
    c->D_all = D; c->T_all = T; c->V = V; c->K = K;
    c->alpha = alpha; c->beta = beta; c->seed = seed;
    c->stream = (hipStream_t)hip_stream;
    int rc = device_limits(c);
    if (rc == MLDA_OK) rc = find_wide_rows(c, word_ids);
    if (rc == MLDA_OK) {
        try { c->chunks = std::vector<HostChunk>(1); } catch (const std::bad_alloc&) { rc = fail(MLDA_ENOMEM, "out of host memory"); }
    }
    if (rc == MLDA_OK) rc = prepare_chunk(doc_ptr, word_ids, 0, D, V, K, false, false, c->run_tiles > 1, c->chunks[0]);
    if (rc == MLDA_OK) rc = check_theta_lds(c, c->chunks[0]);
    if (rc == MLDA_OK) mark_wide_tiles(c, c->chunks[0]);
    const ModelLayout ML = model_layout(V, K, T, false);
    if (rc == MLDA_OK && ML.total + c->chunks[0].L.total > workspace_bytes)
        rc = fail(MLDA_ENOMEM, "workspace has " + std::to_string(workspace_bytes) + " bytes, need " +
                                   std::to_string(ML.total + c->chunks[0].L.total));
    if (rc == MLDA_OK) {
        unsigned char* base = (unsigned char*)dev_workspace;
        HostChunk& h = c->chunks[0];
        c->slot_base[0] = base + ML.total;
        point_at(c, h, c->slot_base[0]);
        hipError_t e = hipSuccess;
        if (h.L.static_bytes > 0)
            e = hipMemcpyAsync(c->slot_base[0], h.arena, h.L.static_bytes, hipMemcpyHostToDevice, c->stream);
        if (e != hipSuccess) rc = fail(MLDA_EHIP, std::string("uploading the corpus: ") + hipGetErrorString(e));
        if (rc == MLDA_OK) { derive_chunk_arrays(c); rc = finish_create(c, base, ML); }
        // the upload reads the host arena until the stream has drained: wait for it before the
        // arena goes, whether or not everything before went well
        e = hipStreamSynchronize(c->stream);
        if (rc == MLDA_OK && e != hipSuccess)
            rc = fail(MLDA_EHIP, std::string("uploading the corpus: ") + hipGetErrorString(e));
        h.release();        // the corpus now lives on the device
    }
    if (rc != MLDA_OK) { destroy(c); return rc; }
    *out = c;
    return MLDA_OK;
}

int mlda_create(mlda_ctx** out, const int64_t* doc_ptr, const int32_t* word_ids, int64_t D,
                int32_t V, int32_t K, double alpha, double beta, uint64_t seed,
                void* dev_workspace, size_t workspace_bytes, void* hip_stream) {
    return create_resident(out, doc_ptr, word_ids, D, V, K, alpha, beta, seed, dev_workspace,
                           workspace_bytes, hip_stream, false);
}

int mlda_create_static(mlda_ctx** out, const int64_t* doc_ptr, const int32_t* word_ids, int64_t D,
                       int32_t V, int32_t K, double alpha, double beta, uint64_t seed, void* hip_stream) {
    return create_resident(out, doc_ptr, word_ids, D, V, K, alpha, beta, seed, nullptr, 0, hip_stream, true);
}

int mlda_create_streamed(mlda_ctx** out, const int64_t* doc_ptr, const int32_t* word_ids, int64_t D,
                         int32_t V, int32_t K, double alpha, double beta, uint64_t seed, int32_t n_chunks,
                         void* dev_workspace, size_t workspace_bytes, void* hip_stream) {
    if (!out) return fail(MLDA_EINVAL, "out is null");
    *out = nullptr;
    RC_TRY(check_corpus(doc_ptr, word_ids, true, D, V, K, alpha, beta));
    if (n_chunks < 1) return fail(MLDA_EINVAL, "n_chunks must be >= 1");
    const int64_t T = doc_ptr[D];
    RC_TRY(check_workspace(dev_workspace, workspace_bytes,
                           streamed_workspace_bound(doc_ptr, D, V, K, n_chunks)));
    RC_TRY(check_device_pointer(dev_workspace));
    mlda_ctx* c = new (std::nothrow) mlda_ctx();
    if (!c) return fail(MLDA_ENOMEM, "out of host memory");
    c->D_all = D; c->T_all = T; c->V = V; c->K = K;
    c->alpha = alpha; c->beta = beta; c->seed = seed;
    c->stream = (hipStream_t)hip_stream;
    c->streamed = true;
    int rc = device_limits(c);
    if (rc == MLDA_OK) rc = find_wide_rows(c, word_ids);
    if (rc == MLDA_OK) {
        try {
            c->chunks = std::vector<HostChunk>((size_t)n_chunks);
            c->z_stored.assign((size_t)n_chunks, nullptr);
        } catch (const std::bad_alloc&) { rc = fail(MLDA_ENOMEM, "out of host memory"); }
    }
    size_t chunk_bytes = 0;
    for (int32_t m = 0; rc == MLDA_OK && m < n_chunks; ++m) {
        rc = prepare_chunk(doc_ptr, word_ids, chunk_first(doc_ptr, D, n_chunks, m),
                           chunk_first(doc_ptr, D, n_chunks, m + 1), V, K, true, true, false, c->chunks[(size_t)m]);
        if (rc == MLDA_OK) rc = check_theta_lds(c, c->chunks[(size_t)m]);
        if (rc == MLDA_OK) mark_wide_tiles(c, c->chunks[(size_t)m]);
        if (rc == MLDA_OK) chunk_bytes = std::max(chunk_bytes, c->chunks[(size_t)m].L.total);
    }
    const ModelLayout ML = model_layout(V, K, T, true);
    if (rc == MLDA_OK && ML.total + 2 * chunk_bytes > workspace_bytes)
        rc = fail(MLDA_ENOMEM, "workspace has " + std::to_string(workspace_bytes) + " bytes, need " +
                                   std::to_string(ML.total + 2 * chunk_bytes));
    auto hip_ok = [&](hipError_t e, const char* what) {
        if (rc == MLDA_OK && e != hipSuccess) rc = fail(MLDA_EHIP, std::string(what) + ": " + hipGetErrorString(e));
    };
    if (rc == MLDA_OK) {
        unsigned char* base = (unsigned char*)dev_workspace;
        c->slot_base[0] = base + ML.total;
        c->slot_base[1] = c->slot_base[0] + chunk_bytes;
        void* zh = nullptr;
        hip_ok(hipHostMalloc(&zh, std::max<size_t>((size_t)T * 2, 1), hipHostMallocDefault), "hipHostMalloc");
        c->z_host = (uint16_t*)zh;
        // every stream at the default priority
        hip_ok(hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking), "hipStreamCreateWithFlags");
        hip_ok(hipStreamCreateWithFlags(&c->down_stream, hipStreamNonBlocking), "hipStreamCreateWithFlags");
        hip_ok(hipEventCreateWithFlags(&c->z_ready, hipEventDisableTiming), "hipEventCreateWithFlags");
        for (int s = 0; s < 2; ++s) {
            hip_ok(hipEventCreateWithFlags(&c->slot_ready[s], hipEventDisableTiming), "hipEventCreateWithFlags");
            hip_ok(hipEventCreateWithFlags(&c->slot_free[s], hipEventDisableTiming), "hipEventCreateWithFlags");
            if (rc == MLDA_OK) hip_ok(hipEventRecord(c->slot_free[s], c->stream), "hipEventRecord");
        }
        for (int32_t m = 0; m < n_chunks; ++m) {
            hip_ok(hipEventCreateWithFlags(&c->z_stored[(size_t)m], hipEventDisableTiming), "hipEventCreateWithFlags");
            if (rc == MLDA_OK) hip_ok(hipEventRecord(c->z_stored[(size_t)m], c->stream), "hipEventRecord");
        }
        if (rc == MLDA_OK) rc = finish_create(c, base, ML);
        if (rc == MLDA_OK) {
            // the documents' term of the log-likelihood never changes
            double doc_term = 0.0;
            const double ka = (double)K * alpha, lg_ka = std::lgamma(ka);
            for (int64_t d = 0; d < D; ++d) doc_term += lg_ka - std::lgamma((double)(doc_ptr[d + 1] - doc_ptr[d]) + ka);
            hip_ok(hipMemcpyAsync(c->ll_scalars + 2, &doc_term, 8, hipMemcpyHostToDevice, c->stream), "hipMemcpyAsync");
            hip_ok(hipStreamSynchronize(c->stream), "hipStreamSynchronize");
        }
    }
    if (rc != MLDA_OK) { destroy(c); return rc; }
    *out = c;
    return MLDA_OK;
}

int mlda_init_random(mlda_ctx* c) {
    if (!c) return fail(MLDA_EINVAL, "null context");
    if (c->streamed) {
        RC_TRY(rebuild_model_streamed(c, true));
    } else {
        if (c->T > 0)
            hipLaunchKernelGGL(mlda::init_topics_kernel, dim3(blocks_for(c->T, 256)), dim3(256), 0,
                               c->stream, c->tok_id, c->z[c->cur], c->T, c->K, c->seed);
        RC_TRY(launch_check("init_topics_kernel"));
        RC_TRY(rebuild_phi(c, c->z[c->cur], 0));
        RC_TRY(rebuild_theta(c, c->z[c->cur]));
    }
    c->iter = 0;
    c->has_state = true;
    c->ll_fresh = false;
    c->last_step_iters = 0;     // the rows of mlda_get_timing / mlda_get_sampler_bytes belong to a step
    c->timed_iters = 0;
    return MLDA_OK;
}

int mlda_set_assignments(mlda_ctx* c, const uint16_t* z, int32_t iter) {
    if (!c) return fail(MLDA_EINVAL, "null context");
    if (c->T_all > 0 && !z) return fail(MLDA_EINVAL, "z is null");
    if (iter < 0) return fail(MLDA_EINVAL, "iter must be >= 0");
    for (int64_t t = 0; t < c->T_all; ++t)
        if (z[t] >= c->K) return fail(MLDA_EINVAL, "topic >= K in z");
    if (c->streamed) {
        HIP_TRY(hipStreamSynchronize(c->stream));
        HIP_TRY(hipStreamSynchronize(c->copy_stream));
        HIP_TRY(hipStreamSynchronize(c->down_stream));
        if (c->T_all > 0) std::memcpy(c->z_host, z, (size_t)c->T_all * 2);
        RC_TRY(rebuild_model_streamed(c, false));
    } else {
        if (c->T > 0) {
            uint16_t* tmp = c->z[c->cur ^ 1];
            HIP_TRY(hipMemcpyAsync(tmp, z, (size_t)c->T * 2, hipMemcpyHostToDevice, c->stream));
            hipLaunchKernelGGL(mlda::to_word_major_kernel, dim3(blocks_for(c->T, 256)), dim3(256), 0,
                               c->stream, tmp, c->tok_id, c->z[c->cur], c->T, (int64_t)0);
            HIP_TRY(hipStreamSynchronize(c->stream));     // the caller's z may go away after return
        }
        RC_TRY(rebuild_phi(c, c->z[c->cur], 0));
        RC_TRY(rebuild_theta(c, c->z[c->cur]));
    }
    c->iter = iter;
    c->has_state = true;
    c->ll_fresh = false;
    c->last_step_iters = 0;
    c->timed_iters = 0;
    return MLDA_OK;
}

// One iteration with several chunks (Algorithm 1, WorkSchedule2; Section 4: every chunk
// samples against the phi of the iteration's start, the new phi is the sum over chunks).
static int step_streamed(mlda_ctx* c, bool loglik, int32_t timed_row) {
    const int next = c->model_cur ^ 1;
    RC_TRY(begin_model(c, next));
    bool first = true;
    for (int32_t m = 0; m < (int32_t)c->chunks.size(); ++m) {
        if (c->chunks[(size_t)m].D == 0) continue;
        hipEvent_t* ev = nullptr;
        if (timed_row >= 0 && (int)c->visit_log.size() < kMaxTimedVisits) {
            const size_t event0 = c->visit_log.size() * kVisitEvents;
            while (c->events.size() < event0 + kVisitEvents) {
                hipEvent_t e;
                HIP_TRY(hipEventCreate(&e));
                c->events.push_back(e);
            }
            ev = &c->events[event0];
        }
        RC_TRY(attach(c, m, true, ev));
        if (ev) {
            try {
                c->visit_log.push_back({timed_row, c->T, c->n_tiles, c->n_wide_tiles, c->rebuilds,
                                        (size_t)(ev - c->events.data())});
            } catch (const std::bad_alloc&) { return fail(MLDA_ENOMEM, "out of host memory"); }
        }
        RC_TRY(rebuild_theta(c, c->z_doc));            // theta is not kept between visits
        if (ev) HIP_TRY(hipEventRecord(ev[2], c->stream));
        RC_TRY(launch_sampler(c, c->z[0], c->z[1]));
        if (ev) HIP_TRY(hipEventRecord(ev[3], c->stream));
        RC_TRY(rebuild_phi(c, c->z[1], next));
        if (ev) HIP_TRY(hipEventRecord(ev[4], c->stream));
        RC_TRY(to_document_order(c, c->z[1]));
        if (ev) HIP_TRY(hipEventRecord(ev[5], c->stream));
        if (loglik) {
            RC_TRY(rebuild_theta(c, c->z_doc));
            RC_TRY(add_theta_loglik(c, first));
            first = false;
        }
        if (ev) HIP_TRY(hipEventRecord(ev[6], c->stream));
        RC_TRY(store_z_and_release(c, m, true));
    }
    RC_TRY(finish_model(c, next));
    c->model_cur = next;
    c->iter += 1;
    c->ll_fresh = false;
    if (loglik) {
        if (first) {
            hipLaunchKernelGGL(mlda::loglik_final_kernel, dim3(1), dim3(256), 0, c->stream, c->ll_partial, 0,
                               (const double*)nullptr, 0, c->ll_scalars + 1);
            RC_TRY(launch_check("loglik_final_kernel"));
        }
        RC_TRY(finish_loglik_streamed(c));
    }
    return MLDA_OK;
}

int mlda_step(mlda_ctx* c, int32_t n_iters, uint32_t flags) {
    RC_TRY(need_state(c));
    if (n_iters < 0) return fail(MLDA_EINVAL, "n_iters must be >= 0");
    if (c->streamed) {
        // the last iterations of the step are timed, as many as the visit log holds
        int32_t visits_per_iter = 0;
        for (const HostChunk& h : c->chunks) visits_per_iter += h.D > 0 ? 1 : 0;
        const int32_t timed = visits_per_iter == 0 ? 0
            : std::min({n_iters, kMaxTimedIters, kMaxTimedVisits / visits_per_iter,
                        kEntryRing / (2 * visits_per_iter) - 1});
        c->visit_log.clear();
        c->timed_iters = std::max(timed, 0);
        c->last_step_iters = n_iters;
        for (int32_t i = 0; i < n_iters; ++i)
            RC_TRY(step_streamed(c, (flags & MLDA_STEP_LOGLIK) != 0, i - (n_iters - c->timed_iters)));
        return MLDA_OK;
    }
    const int32_t timed = std::min(n_iters, kMaxTimedIters);
    while ((int32_t)c->events.size() < timed * 5) {
        hipEvent_t ev;
        HIP_TRY(hipEventCreate(&ev));
        c->events.push_back(ev);
    }
    c->timed_iters = timed;
    c->last_step_iters = n_iters;
    for (int32_t i = 0; i < n_iters; ++i) {
        const int32_t slot = i - (n_iters - timed);
        hipEvent_t* ev = slot >= 0 ? &c->events[(size_t)slot * 5] : nullptr;
        if (ev) HIP_TRY(hipEventRecord(ev[0], c->stream));
        uint16_t* z_next = c->z[c->cur ^ 1];
        RC_TRY(launch_sampler(c, c->z[c->cur], z_next));
        if (ev) HIP_TRY(hipEventRecord(ev[1], c->stream));
        RC_TRY(rebuild_phi(c, z_next, 0));
        if (ev) HIP_TRY(hipEventRecord(ev[2], c->stream));
        RC_TRY(rebuild_theta(c, z_next));
        if (ev) HIP_TRY(hipEventRecord(ev[3], c->stream));
        c->cur ^= 1;
        c->iter += 1;
        c->ll_fresh = false;
        if (flags & MLDA_STEP_LOGLIK) RC_TRY(launch_loglik(c));
        if (ev) HIP_TRY(hipEventRecord(ev[4], c->stream));
    }
    return MLDA_OK;
}

int mlda_iteration(const mlda_ctx* c, int32_t* iter) {
    if (!c || !iter) return fail(MLDA_EINVAL, "null argument");
    *iter = c->iter;
    return MLDA_OK;
}

int mlda_get_assignments(mlda_ctx* c, uint16_t* z) {
    RC_TRY(need_state(c));
    if (c->T_all == 0) return MLDA_OK;
    if (!z) return fail(MLDA_EINVAL, "z is null");
    if (c->streamed) {
        HIP_TRY(hipStreamSynchronize(c->stream));
        HIP_TRY(hipStreamSynchronize(c->down_stream));
        std::memcpy(z, c->z_host, (size_t)c->T_all * 2);
        return MLDA_OK;
    }
    uint16_t* tmp = c->z[c->cur ^ 1];      // free between steps
    hipLaunchKernelGGL(mlda::to_doc_major_scatter_kernel, dim3(blocks_for(c->T, 256)), dim3(256), 0, c->stream,
                       c->z[c->cur], c->tok_id, tmp, c->T, c->at->tok_begin);
    HIP_TRY(hipMemcpyAsync(z, tmp, (size_t)c->T * 2, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return MLDA_OK;
}

int mlda_get_word_topic(mlda_ctx* c, int32_t* n_wk) {
    RC_TRY(need_state(c));
    if (!n_wk) return fail(MLDA_EINVAL, "n_wk is null");
    // the 16-bit matrix and the wide rows are fetched as they are and widened here
    const size_t cells = (size_t)c->V * (size_t)c->K, wide_cells = (size_t)c->n_wide * (size_t)c->K;
    std::vector<uint16_t> narrow;
    std::vector<int32_t> wide;
    try { narrow.resize(cells); wide.resize(wide_cells); }
    catch (const std::bad_alloc&) { return fail(MLDA_ENOMEM, "out of host memory"); }
    const mlda::PhiView& phi = c->phi[c->model_cur];
    HIP_TRY(hipMemcpyAsync(narrow.data(), phi.narrow, cells * 2, hipMemcpyDeviceToHost, c->stream));
    if (wide_cells > 0)
        HIP_TRY(hipMemcpyAsync(wide.data(), phi.wide, wide_cells * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    for (int32_t v = 0; v < c->V; ++v) {
        const int32_t r = c->wide_row[(size_t)v];
        int32_t* row = n_wk + (size_t)v * (size_t)c->K;
        if (r >= 0) std::memcpy(row, wide.data() + (size_t)r * (size_t)c->K, (size_t)c->K * 4);
        else for (int32_t k = 0; k < c->K; ++k) row[k] = narrow[(size_t)v * (size_t)c->K + (size_t)k];
    }
    return MLDA_OK;
}

int mlda_get_topic_totals(mlda_ctx* c, int32_t* n_k) {
    RC_TRY(need_state(c));
    if (!n_k) return fail(MLDA_EINVAL, "n_k is null");
    HIP_TRY(hipMemcpyAsync(n_k, c->n_k[c->model_cur], (size_t)c->K * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return MLDA_OK;
}

int mlda_get_doc_topic_nnz(mlda_ctx* c, int64_t* nnz) {
    RC_TRY(need_state(c));
    if (!nnz) return fail(MLDA_EINVAL, "nnz is null");
    int64_t n = 0;
    std::vector<uint2> rec;
    if (c->streamed) {
        RC_TRY(for_each_chunk_rows(c, [&](const HostChunk&) {
            RC_TRY(fetch_row_rec(c, rec));
            for (const uint2& r : rec) n += r.y;
            return (int)MLDA_OK;
        }));
    } else {
        RC_TRY(fetch_row_rec(c, rec));
        for (const uint2& r : rec) n += r.y;
    }
    *nnz = n;
    return MLDA_OK;
}

int mlda_get_doc_topic_csr(mlda_ctx* c, int64_t* row_ptr, uint16_t* topics, int32_t* counts) {
    RC_TRY(need_state(c));
    if (!row_ptr) return fail(MLDA_EINVAL, "row_ptr is null");
    std::vector<uint2> rec;
    std::vector<unsigned char> slots;
    row_ptr[0] = 0;
    auto take_rows = [&](const HostChunk& h) {
        RC_TRY(fetch_rows(c, rec, slots));
        int64_t* ptr = row_ptr + h.d_begin;
        for (int64_t d = 0; d < c->D; ++d) ptr[d + 1] = ptr[d] + rec[(size_t)d].y;
        if (ptr[c->D] > ptr[0] && (!topics || !counts)) return fail(MLDA_EINVAL, "topics or counts is null");
        unpack_rows(c, rec, slots, ptr, topics, counts);
        return (int)MLDA_OK;
    };
    if (c->streamed) {
        // chunks are visited in document order, so every chunk finds its first row start in place
        RC_TRY(for_each_chunk_rows(c, take_rows));
    } else {
        RC_TRY(take_rows(c->chunks[0]));
    }
    return MLDA_OK;
}

int mlda_get_loglik(mlda_ctx* c, double* ll) {
    RC_TRY(need_state(c));
    if (!ll) return fail(MLDA_EINVAL, "ll is null");
    if (!c->ll_fresh) {
        if (c->streamed) {
            RC_TRY(for_each_chunk_rows(c, [](const HostChunk&) { return (int)MLDA_OK; }));
            RC_TRY(finish_loglik_streamed(c));
        } else {
            RC_TRY(launch_loglik(c));
        }
    }
    HIP_TRY(hipMemcpyAsync(ll, c->ll_scalars, 8, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return MLDA_OK;
}

int mlda_get_timing(mlda_ctx* c, double* ms, int32_t capacity_iters, int32_t* n_iters) {
    if (!c || !ms || !n_iters || capacity_iters < 0) return fail(MLDA_EINVAL, "bad argument");
    HIP_TRY(hipStreamSynchronize(c->stream));
    const int32_t n = std::min(c->timed_iters, capacity_iters);
    const int32_t first = c->timed_iters - n;
    if (c->streamed) {
        // per iteration the sums over its chunk visits: sampling | phi | theta rebuild and the
        // two order changes | the theta rebuild of the new topics (log-likelihood)
        HIP_TRY(hipStreamSynchronize(c->down_stream));
        for (int32_t i = 0; i < 4 * n; ++i) ms[i] = 0.0;
        for (const mlda_ctx::Visit& v : c->visit_log) {
            if (v.iter_row < first) continue;
            hipEvent_t* ev = &c->events[v.event0];
            float t[kVisitEvents - 1];
            for (int j = 0; j + 1 < kVisitEvents; ++j) HIP_TRY(hipEventElapsedTime(&t[j], ev[j], ev[j + 1]));
            double* row = ms + (size_t)(v.iter_row - first) * 4;
            row[0] += t[2];
            row[1] += t[3];
            row[2] += t[0] + t[1] + t[4];
            row[3] += t[5];
        }
        *n_iters = n;
        return MLDA_OK;
    }
    for (int32_t i = 0; i < n; ++i) {
        hipEvent_t* ev = &c->events[(size_t)(first + i) * 5];
        for (int j = 0; j < 4; ++j) {
            float t = 0.f;
            HIP_TRY(hipEventElapsedTime(&t, ev[j], ev[j + 1]));
            ms[(size_t)i * 4 + j] = (double)t;
        }
    }
    *n_iters = n;
    return MLDA_OK;
}

int mlda_get_sampler_bytes(mlda_ctx* c, double* bytes, int32_t capacity_iters, int32_t* n_iters) {
    RC_TRY(need_state(c));
    if (!bytes || !n_iters || capacity_iters < 0) return fail(MLDA_EINVAL, "bad argument");
    const int32_t n = std::min({c->last_step_iters, capacity_iters, kMaxTimedIters});
    // iteration j of the step (0-based, of last_step_iters) sampled from the state left by
    // rebuild number (rebuilds - last_step_iters + j - 1)
    std::vector<unsigned long long> ring((size_t)kEntryRing);
    HIP_TRY(hipMemcpyAsync(ring.data(), c->row_entries, (size_t)kEntryRing * 8, hipMemcpyDeviceToHost,
                           c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    const double entry_bytes = tiny_rows_for(c->K) ? 2.0 : 4.0;
    if (c->streamed) {          // per iteration the sum over its chunk visits
        const int32_t m = std::min(c->timed_iters, capacity_iters), first = c->timed_iters - m;
        for (int32_t i = 0; i < m; ++i) bytes[i] = 0.0;
        for (const mlda_ctx::Visit& v : c->visit_log) {
            if (v.iter_row < first) continue;
            bytes[v.iter_row - first] += 16.0 * (double)v.T +
                entry_bytes * (double)ring[(size_t)(v.rebuild % kEntryRing)] +
                (double)c->K * (2.0 * (double)v.n_tiles + 2.0 * (double)v.n_wide_tiles);
        }
        *n_iters = m;
        return MLDA_OK;
    }
    for (int32_t i = 0; i < n; ++i) {
        const int32_t j = c->last_step_iters - n + i;
        const int64_t r = c->rebuilds - c->last_step_iters + j - 1;
        const double row_entries = c->D > 0 ? (double)ring[(size_t)(r % kEntryRing)] : 0.0;
        // per token: row slot 4, token id 4, old topic 2, new topic 2, row length 4
        // per tile: the word's row of phi, 2 K bytes, or 4 K for a word with 2^16 tokens or more;
        // a tile that follows another in a run reads, instead of a row of phi, the topics of
        // the previous tile's tokens and, for its own tokens, topic and cell of phi: 6 bytes
        // per token, counted as if both tiles had this tile's tokens
        const int32_t n_run_tiles = c->run_tiles > 1 ? c->n_tiles - c->n_single : 0;
        const int32_t n_runs = n_run_tiles > 0 ? (n_run_tiles + c->run_tiles - 1) / c->run_tiles : 0;
        const double staged_rows = (double)(c->n_tiles - n_run_tiles + n_runs);
        bytes[i] = 16.0 * (double)c->T + entry_bytes * row_entries +
                   (double)c->K * (2.0 * staged_rows + 2.0 * (double)c->n_wide_tiles) +
                   6.0 * (double)c->run_tokens;
    }
    *n_iters = n;
    return MLDA_OK;
}

void mlda_destroy(mlda_ctx* c) { destroy(c); }

int mlda_philox_uniform(uint64_t seed, uint32_t iter, uint64_t token0, int64_t n, double* out_dev,
                        void* hip_stream) {
    if (n < 0) return fail(MLDA_EINVAL, "n must be >= 0");
    if (n == 0) return MLDA_OK;
    if (!out_dev) return fail(MLDA_EINVAL, "out_dev is null");
    hipLaunchKernelGGL(mlda::philox_uniform_kernel, dim3(blocks_for(n, 256)), dim3(256), 0,
                       (hipStream_t)hip_stream, seed, iter, token0, n, out_dev);
    return launch_check("philox_uniform_kernel");
}

}  // extern "C"
