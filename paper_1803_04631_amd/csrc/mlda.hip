// libmlda.so: C ABI, context and host-side preprocessing (see include/mlda.h).
//
// Paper sections behind the host steps: Section 6.1.2 (tokens are sorted word-first and
// the tokens of heavy words are split over several workgroups that are issued first),
// Section 6.2 (a document->token map built on the CPU lets the theta update find a
// document's tokens in the word-sorted arrays), Algorithm 1 WorkSchedule1 with one
// chunk on one GPU (transfer once, then iterate on the device).
#include "../../include/mlda.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
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

constexpr size_t kAlign = 256;        // workspace sub-buffer alignment
constexpr size_t kSlotAlign = 64;     // theta row slot alignment (bytes)
// waves per sampling workgroup: more of them share one staged p* column when K is large
int sample_waves_for(int32_t K) { return K <= 2048 ? 4 : 16; }

const void* sample_kernel_for(int32_t K, bool packed) {
    if (sample_waves_for(K) == 4)
        return packed ? (const void*)mlda::sample_kernel<4, mlda::PackedRows>
                      : (const void*)mlda::sample_kernel<4, mlda::SplitRows>;
    return packed ? (const void*)mlda::sample_kernel<16, mlda::PackedRows>
                  : (const void*)mlda::sample_kernel<16, mlda::SplitRows>;
}
constexpr int kMaxTimedIters = 1024;

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int tile_tokens_for(int32_t K) { return K <= 2048 ? 1024 : 4096; }
constexpr int kPhiSegment = 16384;    // tokens one workgroup histograms for the phi rebuild

// A theta row's slot: a header of kRowHeader bytes (the row's length), then the entries.
size_t slot_bytes_for(int64_t cap, int entry_bytes) {   // cap = largest nnz the row can reach
    return align_up((size_t)mlda::kRowHeader + (size_t)(((cap + 3) & ~(int64_t)3) * entry_bytes),
                    kSlotAlign);
}

// Sizes of every workspace sub-buffer, as upper bounds from (D, T, V, K) or exactly.
struct Layout {
    size_t tok_slot, tok_id, doc_map, z0, z1, doc_ptr, doc_order, row_rec, slots, n_wk, n_k, tiles, segs, split,
        ll_partial, ll_value, lg_table, row_entries, total;
    void finish() {
        size_t* parts[] = {&tok_slot, &tok_id, &doc_map, &z0, &z1, &doc_ptr, &doc_order, &row_rec, &slots,
                           &n_wk, &n_k, &tiles, &segs, &split, &ll_partial, &ll_value, &lg_table, &row_entries};
        total = 0;
        for (size_t* p : parts) { *p = align_up(*p, kAlign); total += *p; }
    }
};

constexpr int kLoglikBlocks = 2048;
constexpr int kMaxThetaGrid = 8192;    // workgroups of the theta rebuild (each leaves one likelihood partial)
constexpr int kEntryRing = 2048;      // per-rebuild counters of theta row entries (> kMaxTimedIters)

Layout layout_for(int64_t D, int64_t T, int32_t V, int32_t K, size_t slots_bytes, size_t n_tiles,
                  size_t n_segs, size_t n_split) {
    Layout L{};
    L.tok_slot = (size_t)T * 4;
    L.tok_id = (size_t)T * 4;
    L.doc_map = (size_t)T * 4;
    L.z0 = (size_t)T * 2;
    L.z1 = (size_t)T * 2;
    L.doc_ptr = (size_t)(D + 1) * 4;
    L.doc_order = (size_t)D * sizeof(mlda::DocRec);
    L.row_rec = (size_t)D * 8;
    L.slots = slots_bytes;
    L.n_wk = (size_t)V * (size_t)K * 4;
    L.n_k = (size_t)K * 4;
    L.tiles = n_tiles * sizeof(mlda::Tile);
    L.segs = n_segs * sizeof(mlda::Tile);
    L.split = n_split * 4;
    L.ll_partial = (size_t)(2 * kLoglikBlocks + kMaxThetaGrid) * 8;
    L.ll_value = 8;
    L.lg_table = (size_t)(mlda::kLgTable + 1) * 8 * 2;     // one for alpha, one for beta
    L.row_entries = (size_t)kEntryRing * 8;
    L.finish();
    return L;
}

Layout layout_bound(int64_t D, int64_t T, int32_t V, int32_t K) {
    const size_t tile = (size_t)tile_tokens_for(K);
    const size_t slots = kSlotAlign + (size_t)T * 6 + (size_t)D * (mlda::kRowHeader + 18 + kSlotAlign);
    const size_t n_tiles = (size_t)T / tile + (size_t)V + 1;
    const size_t n_segs = (size_t)T / kPhiSegment + (size_t)V + 1;
    return layout_for(D, T, V, K, slots, n_tiles, n_segs, (size_t)V);
}

template <class F>
void parallel_chunks(int n_chunks, F&& body) {
    std::vector<std::thread> pool;
    for (int c = 1; c < n_chunks; ++c) pool.emplace_back([&, c] { body(c); });
    body(0);
    for (auto& t : pool) t.join();
}

}  // namespace

struct mlda_ctx {
    int64_t D = 0, T = 0;
    int32_t V = 0, K = 0, Kpad = 0;
    double alpha = 0, beta = 0;
    uint64_t seed = 0;
    int32_t iter = 0;
    hipStream_t stream = nullptr;
    int n_cus = 0, lds_limit = 0;

    uint32_t* tok_slot = nullptr;         // [T] slot of the theta row of each word-major token's document
    int32_t *tok_id = nullptr, *doc_map = nullptr, *doc_ptr = nullptr;
    mlda::DocRec* doc_order = nullptr;  // documents by falling length, as the theta rebuild walks them
    int32_t theta_grid = 0;
    bool packed = false;                // theta rows as 4-byte entries (no document has 2^14 tokens)
    int32_t *n_wk = nullptr, *n_k = nullptr, *split_words = nullptr;
    uint16_t* z[2] = {nullptr, nullptr};
    int cur = 0;
    uint2* row_rec = nullptr;
    unsigned char* slots = nullptr;
    size_t slots_bytes = 0;
    mlda::Tile* tiles = nullptr;        // sampling tiles
    mlda::Tile* segs = nullptr;         // phi rebuild segments
    int32_t n_tiles = 0, n_segs = 0, n_split = 0;
    double *ll_partial = nullptr, *ll_value = nullptr;
    double* lg_table = nullptr;          // lgG(c + alpha) - lgG(alpha), c < 1024, then lgG(alpha)
    double* lg_table_beta = nullptr;     // the same for beta
    unsigned long long* row_entries = nullptr;   // ring: [r % kEntryRing] written by rebuild r
    int64_t rebuilds = 0;                        // rebuilds launched so far
    int32_t last_step_iters = 0;

    std::vector<int64_t> doc_ptr_host;
    bool has_state = false, ll_fresh = false;

    std::vector<hipEvent_t> events;     // 5 per timed iteration
    int32_t timed_iters = 0;            // iterations of the last step that carry events
    size_t sample_lds = 0;
};

namespace {

int launch_check(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(MLDA_EHIP, std::string(what) + ": " + hipGetErrorString(e));
    return MLDA_OK;
}

int blocks_for(int64_t n, int per) { return (int)((n + per - 1) / per); }

// phi, n_k and theta from the assignments in z (word-major).  ev: optional events
// [after phi+n_k, after theta].
int rebuild_counts(mlda_ctx* c, const uint16_t* z, hipEvent_t* ev_phi, hipEvent_t* ev_theta) {
    using namespace mlda;
    const size_t hist_bytes = (size_t)c->K * 4;
    if (c->n_split > 0) {
        dim3 grid((unsigned)c->n_split, (unsigned)blocks_for(c->K, 256));
        hipLaunchKernelGGL(zero_rows_kernel, grid, dim3(256), 0, c->stream, c->split_words, c->n_wk,
                           c->K);
    }
    hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks_for(c->K, 256)), dim3(256), 0, c->stream, c->n_k,
                       (int64_t)c->K, 0);
    if (c->n_tiles > 0) {
        hipLaunchKernelGGL(phi_tile_kernel, dim3((unsigned)c->n_segs), dim3(256), hist_bytes,
                           c->stream, c->segs, z, c->n_wk, c->K);
        if ((int64_t)c->V * c->K * 2 < c->T) {
            // n_k as column sums of the fresh n_wk: fewer bytes than z and no LDS atomics
            const int words_per_slice = 64;
            dim3 grid((unsigned)blocks_for(c->K, 256), (unsigned)blocks_for(c->V, words_per_slice));
            hipLaunchKernelGGL(topic_totals_from_rows_kernel, grid, dim3(256), 0, c->stream, c->n_wk,
                               c->V, c->K, words_per_slice, c->n_k);
        } else {
            const int grid = (int)std::min<int64_t>((c->T + 4095) / 4096, (int64_t)c->n_cus * 8);
            hipLaunchKernelGGL(topic_totals_kernel, dim3((unsigned)grid), dim3(256), hist_bytes,
                               c->stream, z, c->T, c->n_k, c->K);
        }
    }
    if (ev_phi) HIP_TRY(hipEventRecord(*ev_phi, c->stream));
    if (c->D > 0) {
        const size_t theta_lds = theta_lds_bytes(c->K, c->packed);
        unsigned long long* entries = c->row_entries + (c->rebuilds % kEntryRing);
        hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, c->stream, entries);
        if (c->packed)
            hipLaunchKernelGGL(theta_rows_kernel<true>, dim3((unsigned)c->theta_grid), dim3(kWave),
                               theta_lds, c->stream, c->doc_order, c->doc_map, z, c->row_rec, c->slots,
                               c->D, c->K, c->alpha, c->lg_table, entries,
                               c->ll_partial + 2 * kLoglikBlocks);
        else
            hipLaunchKernelGGL(theta_rows_kernel<false>, dim3((unsigned)c->theta_grid), dim3(kWave),
                               theta_lds, c->stream, c->doc_order, c->doc_map, z, c->row_rec, c->slots,
                               c->D, c->K, c->alpha, c->lg_table, entries,
                               c->ll_partial + 2 * kLoglikBlocks);
    }
    c->rebuilds += 1;
    if (ev_theta) HIP_TRY(hipEventRecord(*ev_theta, c->stream));
    return launch_check("rebuild kernels");
}

int launch_loglik(mlda_ctx* c) {
    using namespace mlda;
    const int64_t cells = (int64_t)c->V * c->K;
    hipLaunchKernelGGL(loglik_word_side_kernel, dim3(kLoglikBlocks), dim3(256), 0, c->stream, c->n_wk,
                       cells, c->n_k, c->K, c->beta, (double)c->V * c->beta, c->lg_table_beta,
                       c->ll_partial);
    hipLaunchKernelGGL(loglik_doc_term_kernel, dim3(kLoglikBlocks), dim3(256), 0, c->stream,
                       c->doc_ptr, c->D, (double)c->K * c->alpha, c->ll_partial + kLoglikBlocks);
    hipLaunchKernelGGL(loglik_final_kernel, dim3(1), dim3(256), 0, c->stream, c->ll_partial,
                       2 * kLoglikBlocks + c->theta_grid, c->ll_value);
    c->ll_fresh = true;
    return launch_check("log-likelihood kernels");
}

int need_state(const mlda_ctx* c) {
    if (!c) return fail(MLDA_EINVAL, "null context");
    if (!c->has_state)
        return fail(MLDA_EINVAL, "no topic assignments yet: call mlda_init_random or mlda_set_assignments");
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
        case MLDA_ENOTSUP: return "K too large for the device's LDS";
        default: return "unknown error";
    }
}

const char* mlda_last_error(void) { return g_last_error.c_str(); }

int mlda_workspace_bytes(int64_t D, int64_t T, int32_t V, int32_t K, size_t* bytes) {
    if (!bytes) return fail(MLDA_EINVAL, "bytes is null");
    if (D < 0 || T < 0 || V < 1 || K < 1 || K > 65535 || T >= ((int64_t)1 << 31))
        return fail(MLDA_EINVAL, "need D >= 0, 0 <= T < 2^31, V >= 1, 1 <= K <= 65535");
    *bytes = layout_bound(D, T, V, K).total;
    return MLDA_OK;
}

int mlda_create(mlda_ctx** out, const int64_t* doc_ptr, const int32_t* word_ids, int64_t D,
                int32_t V, int32_t K, double alpha, double beta, uint64_t seed,
                void* dev_workspace, size_t workspace_bytes, void* hip_stream) {
    if (!out) return fail(MLDA_EINVAL, "out is null");
    *out = nullptr;
    if (!doc_ptr) return fail(MLDA_EINVAL, "doc_ptr is null");
    if (D < 0 || V < 1) return fail(MLDA_EINVAL, "need D >= 0 and V >= 1");
    if (K < 1 || K > 65535) return fail(MLDA_EINVAL, "K must be in [1, 65535] (16-bit topic indices)");
    if (!(alpha > 0.0) || !(beta > 0.0) || !std::isfinite(alpha) || !std::isfinite(beta))
        return fail(MLDA_EINVAL, "alpha and beta must be positive and finite");
    if (doc_ptr[0] != 0) return fail(MLDA_EINVAL, "doc_ptr[0] must be 0");
    for (int64_t d = 0; d < D; ++d)
        if (doc_ptr[d + 1] < doc_ptr[d]) return fail(MLDA_EINVAL, "doc_ptr must be non-decreasing");
    const int64_t T = doc_ptr[D];
    if (T >= ((int64_t)1 << 31)) return fail(MLDA_EINVAL, "2^31 or more tokens");
    if (T > 0 && !word_ids) return fail(MLDA_EINVAL, "word_ids is null");
    if (!dev_workspace) return fail(MLDA_EINVAL, "dev_workspace is null");
    if (((uintptr_t)dev_workspace) % kAlign != 0)
        return fail(MLDA_EINVAL, "dev_workspace must be 256-byte aligned");
    size_t need_bound = 0;
    if (mlda_workspace_bytes(D, T, V, K, &need_bound) != MLDA_OK) return MLDA_EINVAL;
    if (workspace_bytes < need_bound)
        return fail(MLDA_ENOMEM, "workspace has " + std::to_string(workspace_bytes) + " bytes, need " +
                                     std::to_string(need_bound));
    {
        hipPointerAttribute_t attr;
        hipError_t e = hipPointerGetAttributes(&attr, dev_workspace);
        if (e != hipSuccess || attr.type != hipMemoryTypeDevice) {
            (void)hipGetLastError();
            return fail(MLDA_EINVAL, "dev_workspace is not device memory");
        }
    }

    int dev = 0, n_cus = 0, lds_limit = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&n_cus, hipDeviceAttributeMultiprocessorCount, dev));
    HIP_TRY(hipDeviceGetAttribute(&lds_limit, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
    // one zero entry of p* past the last topic: padding entries of theta rows point at it
    const int32_t dense_group = mlda::dense_group(sample_waves_for(K));
    const int32_t Kpad = (K + dense_group) / dense_group * dense_group;
    const size_t sample_lds = mlda::sample_lds_bytes(Kpad, sample_waves_for(K));
    if (sample_lds > (size_t)lds_limit)
        return fail(MLDA_ENOTSUP, "K = " + std::to_string(K) + " needs " + std::to_string(sample_lds) +
                                      " bytes of LDS per workgroup, the device allows " +
                                      std::to_string(lds_limit));

    // ---- word-first order (Section 6.1.2).  Inside a word the tokens are put in order of
    // falling document length, so that the four theta rows a wave walks together have
    // similar lengths; any order inside a word gives the same result, because the uniforms
    // are keyed by the caller's token index.  Stable counting sort by word over chunks of
    // the length-sorted document sequence.
    int64_t longest_doc = 0;
    for (int64_t d = 0; d < D; ++d) longest_doc = std::max(longest_doc, doc_ptr[d + 1] - doc_ptr[d]);
    // a count never exceeds the document's length: 4-byte theta entries if 14 bits hold it
    const bool packed = longest_doc <= mlda::PackedRows::kMaxCount;
    const int entry_bytes = packed ? mlda::PackedRows::kEntryBytes : mlda::SplitRows::kEntryBytes;
    std::vector<int32_t> doc_order;
    std::vector<int64_t> order_tokens;           // tokens before each position of doc_order
    try {
        doc_order.resize((size_t)D);
        order_tokens.resize((size_t)D + 1);
        const int64_t max_len = longest_doc;
        std::vector<int64_t> len_start((size_t)max_len + 2, 0);
        for (int64_t d = 0; d < D; ++d) ++len_start[(size_t)(max_len - (doc_ptr[d + 1] - doc_ptr[d])) + 1];
        for (int64_t l = 0; l <= max_len; ++l) len_start[(size_t)l + 1] += len_start[(size_t)l];
        for (int64_t d = 0; d < D; ++d)
            doc_order[(size_t)len_start[(size_t)(max_len - (doc_ptr[d + 1] - doc_ptr[d]))]++] = (int32_t)d;
        order_tokens[0] = 0;
        for (int64_t i = 0; i < D; ++i) {
            const int64_t d = doc_order[(size_t)i];
            order_tokens[(size_t)i + 1] = order_tokens[(size_t)i] + (doc_ptr[d + 1] - doc_ptr[d]);
        }
    } catch (const std::bad_alloc&) {
        return fail(MLDA_ENOMEM, "out of host memory");
    }
    const int n_chunks = (int)std::max<int64_t>(
        1, std::min<int64_t>({(int64_t)std::thread::hardware_concurrency(), 32, T / 65536 + 1}));
    std::vector<std::vector<int32_t>> chunk_hist(n_chunks);
    std::vector<int> chunk_bad(n_chunks, 0);
    // chunk c holds the documents doc_order[chunk_lo(c) .. chunk_lo(c+1)), about T/n_chunks tokens
    auto chunk_lo = [&](int c) -> int64_t {
        if (c >= n_chunks) return D;
        const int64_t want = T / n_chunks * c;
        return std::lower_bound(order_tokens.begin(), order_tokens.end(), want) - order_tokens.begin();
    };
    try {
        parallel_chunks(n_chunks, [&](int c) {
            auto& h = chunk_hist[c];
            h.assign((size_t)V, 0);
            for (int64_t i = chunk_lo(c); i < chunk_lo(c + 1); ++i) {
                const int64_t d = doc_order[(size_t)i];
                for (int64_t t = doc_ptr[d]; t < doc_ptr[d + 1]; ++t) {
                    const int32_t w = word_ids[t];
                    if (w < 0 || w >= V) { chunk_bad[c] = 1; return; }
                    ++h[w];
                }
            }
        });
    } catch (const std::bad_alloc&) {
        return fail(MLDA_ENOMEM, "out of host memory");
    }
    for (int c = 0; c < n_chunks; ++c)
        if (chunk_bad[c]) return fail(MLDA_EINVAL, "word id outside [0, V)");

    std::vector<uint32_t> tok_slot;
    std::vector<int32_t> word_ptr((size_t)V + 1, 0), tok_id, doc_map, doc_ptr32, split_words;
    std::vector<uint2> row_rec;
    std::vector<mlda::DocRec> doc_recs;
    std::vector<mlda::Tile> tiles, segs;
    size_t slots_bytes = 0;
    try {
        for (int32_t v = 0; v < V; ++v) {
            int32_t n = 0;
            for (int c = 0; c < n_chunks; ++c) {
                const int32_t h = chunk_hist[c][v];
                chunk_hist[c][v] = n;          // becomes the chunk's offset inside the word
                n += h;
            }
            word_ptr[v + 1] = word_ptr[v] + n;
        }
        // ---- theta row slots: fixed capacity min(N_d, K), so rows never move; laid out in the
        // order the documents are worked on, so that rows in use together are neighbours
        row_rec.resize((size_t)D);
        slots_bytes = kSlotAlign;       // the buffer starts with four padding entries
        for (int64_t i = 0; i < D; ++i) {
            const int64_t d = doc_order[(size_t)i];
            const int64_t cap = std::min<int64_t>(doc_ptr[d + 1] - doc_ptr[d], K);
            if (slots_bytes / 16 > 0xffffffffull)
                return fail(MLDA_ENOTSUP, "theta rows need more than 64 GiB");
            row_rec[(size_t)d] = make_uint2((uint32_t)(slots_bytes / 16), 0u);
            slots_bytes += slot_bytes_for(cap, entry_bytes);
        }
        tok_slot.resize((size_t)T);
        tok_id.resize((size_t)T);
        doc_map.resize((size_t)T);
        parallel_chunks(n_chunks, [&](int c) {
            auto& start = chunk_hist[c];
            for (int64_t i = chunk_lo(c); i < chunk_lo(c + 1); ++i) {
                const int64_t d = doc_order[(size_t)i];
                for (int64_t t = doc_ptr[d]; t < doc_ptr[d + 1]; ++t) {
                    const int32_t w = word_ids[t];
                    const int32_t pos = word_ptr[w] + start[w]++;
                    tok_id[pos] = (int32_t)t;
                    tok_slot[pos] = row_rec[(size_t)d].x;
                    doc_map[t] = pos;
                }
            }
        });
        chunk_hist.clear();

        doc_ptr32.resize((size_t)D + 1);
        for (int64_t d = 0; d <= D; ++d) doc_ptr32[d] = (int32_t)doc_ptr[d];

        doc_recs.resize((size_t)D);
        for (int64_t i = 0; i < D; ++i) {
            const int64_t d = doc_order[(size_t)i];
            doc_recs[(size_t)i] = mlda::DocRec{(int32_t)doc_ptr[d], (int32_t)(doc_ptr[d + 1] - doc_ptr[d]),
                                              row_rec[(size_t)d].x, (int32_t)d};
        }

        // ---- tiles of one word each, largest first (Section 6.1.2)
        const int32_t tile = tile_tokens_for(K);
        for (int32_t v = 0; v < V; ++v) {
            const int32_t n = word_ptr[v + 1] - word_ptr[v];
            for (int32_t b = 0; b < n; b += tile)
                tiles.push_back(mlda::Tile{v, word_ptr[v] + b, std::min(tile, n - b), n <= tile ? 1 : 0});
            if (n > kPhiSegment) split_words.push_back(v);
            for (int32_t b = 0; b < n; b += kPhiSegment)
                segs.push_back(mlda::Tile{v, word_ptr[v] + b, std::min(kPhiSegment, n - b),
                                          n <= kPhiSegment ? 1 : 0});
        }
        auto larger_first = [](const mlda::Tile& a, const mlda::Tile& b) { return a.count > b.count; };
        // Sampling tiles run in the order of their first document (longest documents first),
        // not word by word: tiles of different words that are in flight together then walk the
        // theta rows of the same documents, which are fetched from HBM once instead of once
        // per heavy word.  (The paper issues the tiles of heavy words first, Section 6.1.2;
        // here the long-row tiles come first, which also keeps the tail short.)
        // (slot offsets rise in that order)
        std::stable_sort(tiles.begin(), tiles.end(), [&](const mlda::Tile& a, const mlda::Tile& b) {
            return tok_slot[(size_t)a.begin] < tok_slot[(size_t)b.begin];
        });
        std::stable_sort(segs.begin(), segs.end(), larger_first);
    } catch (const std::bad_alloc&) {
        return fail(MLDA_ENOMEM, "out of host memory");
    }

    const Layout L = layout_for(D, T, V, K, slots_bytes, tiles.size(), segs.size(), split_words.size());
    if (L.total > workspace_bytes)
        return fail(MLDA_ENOMEM, "workspace has " + std::to_string(workspace_bytes) + " bytes, need " +
                                     std::to_string(L.total));

    mlda_ctx* c = new (std::nothrow) mlda_ctx();
    if (!c) return fail(MLDA_ENOMEM, "out of host memory");
    c->D = D; c->T = T; c->V = V; c->K = K; c->Kpad = Kpad;
    c->alpha = alpha; c->beta = beta; c->seed = seed;
    c->stream = (hipStream_t)hip_stream;
    c->n_cus = n_cus; c->lds_limit = lds_limit; c->sample_lds = sample_lds;
    c->n_tiles = (int32_t)tiles.size();
    c->packed = packed;
    {
        const size_t theta_lds = mlda::theta_lds_bytes(K, packed);
        // 16 one-wave workgroups per CU: enough to hide the gathers' latency; more of them
        // touch more lines of z at once than an XCD's L2 holds, and neighbours stop sharing
        const int per_cu = std::max(1, std::min(16, (int)(144 * 1024 / theta_lds)));
        c->theta_grid = (int32_t)std::min<int64_t>({D, (int64_t)n_cus * per_cu, (int64_t)kMaxThetaGrid});
    }
    c->n_segs = (int32_t)segs.size();
    c->n_split = (int32_t)split_words.size();
    c->slots_bytes = slots_bytes;
    c->doc_ptr_host.assign(doc_ptr, doc_ptr + D + 1);

    unsigned char* p = (unsigned char*)dev_workspace;
    auto take = [&](size_t bytes) { unsigned char* q = p; p += bytes; return q; };
    c->tok_slot = (uint32_t*)take(L.tok_slot);
    c->tok_id = (int32_t*)take(L.tok_id);
    c->doc_map = (int32_t*)take(L.doc_map);
    c->z[0] = (uint16_t*)take(L.z0);
    c->z[1] = (uint16_t*)take(L.z1);
    c->doc_ptr = (int32_t*)take(L.doc_ptr);
    c->doc_order = (mlda::DocRec*)take(L.doc_order);
    c->row_rec = (uint2*)take(L.row_rec);
    c->slots = take(L.slots);
    c->n_wk = (int32_t*)take(L.n_wk);
    c->n_k = (int32_t*)take(L.n_k);
    c->tiles = (mlda::Tile*)take(L.tiles);
    c->segs = (mlda::Tile*)take(L.segs);
    c->split_words = (int32_t*)take(L.split);
    c->ll_partial = (double*)take(L.ll_partial);
    c->ll_value = (double*)take(L.ll_value);
    c->lg_table = (double*)take(L.lg_table);
    c->lg_table_beta = c->lg_table + (mlda::kLgTable + 1);
    c->row_entries = (unsigned long long*)take(L.row_entries);

    auto up = [&](void* dst, const void* src, size_t bytes) -> hipError_t {
        if (bytes == 0) return hipSuccess;
        return hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, c->stream);
    };
    hipError_t e = hipSuccess;
    if (e == hipSuccess) e = up(c->tok_slot, tok_slot.data(), (size_t)T * 4);
    if (e == hipSuccess) e = up(c->tok_id, tok_id.data(), (size_t)T * 4);
    if (e == hipSuccess) e = up(c->doc_map, doc_map.data(), (size_t)T * 4);
    if (e == hipSuccess) e = up(c->doc_ptr, doc_ptr32.data(), (size_t)(D + 1) * 4);
    if (e == hipSuccess) e = up(c->doc_order, doc_recs.data(), (size_t)D * sizeof(mlda::DocRec));
    if (e == hipSuccess) e = up(c->row_rec, row_rec.data(), (size_t)D * 8);
    // what a lane of the sampler reads when it has no entries of its own (count 0, topic K)
    const uint32_t pad_entries[4] = {(uint32_t)K << 2, (uint32_t)K << 2, (uint32_t)K << 2, (uint32_t)K << 2};
    if (e == hipSuccess) e = up(c->slots, pad_entries, sizeof(pad_entries));
    if (e == hipSuccess) e = up(c->tiles, tiles.data(), tiles.size() * sizeof(mlda::Tile));
    if (e == hipSuccess) e = up(c->segs, segs.data(), segs.size() * sizeof(mlda::Tile));
    if (e == hipSuccess) e = up(c->split_words, split_words.data(), split_words.size() * 4);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(mlda::lg_table_kernel, dim3(blocks_for(mlda::kLgTable + 1, 256)), dim3(256), 0,
                           c->stream, c->lg_table, alpha);
        hipLaunchKernelGGL(mlda::lg_table_kernel, dim3(blocks_for(mlda::kLgTable + 1, 256)), dim3(256), 0,
                           c->stream, c->lg_table_beta, beta);
        // rows of words without tokens are never written again: start phi at zero
        const int64_t cells = (int64_t)V * K;
        hipLaunchKernelGGL(mlda::fill_i32_kernel, dim3(blocks_for(cells, 256)), dim3(256), 0, c->stream,
                           c->n_wk, cells, 0);
        e = hipGetLastError();
    }
    if (e == hipSuccess && sample_lds > 48 * 1024)
        e = hipFuncSetAttribute(sample_kernel_for(K, packed),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)sample_lds);
    if (e == hipSuccess && (size_t)K * 4 > 48 * 1024) {
        e = hipFuncSetAttribute((const void*)mlda::phi_tile_kernel,
                                hipFuncAttributeMaxDynamicSharedMemorySize, K * 4);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void*)mlda::topic_totals_kernel,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, K * 4);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(packed ? (const void*)mlda::theta_rows_kernel<true>
                                           : (const void*)mlda::theta_rows_kernel<false>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)mlda::theta_lds_bytes(K, packed));
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) {
        delete c;
        return fail(MLDA_EHIP, std::string("uploading the corpus: ") + hipGetErrorString(e));
    }
    *out = c;
    return MLDA_OK;
}

int mlda_init_random(mlda_ctx* c) {
    if (!c) return fail(MLDA_EINVAL, "null context");
    if (c->T > 0)
        hipLaunchKernelGGL(mlda::init_topics_kernel, dim3(blocks_for(c->T, 256)), dim3(256), 0,
                           c->stream, c->tok_id, c->z[c->cur], c->T, c->K, c->seed);
    int rc = launch_check("init_topics_kernel");
    if (rc != MLDA_OK) return rc;
    rc = rebuild_counts(c, c->z[c->cur], nullptr, nullptr);
    if (rc != MLDA_OK) return rc;
    c->iter = 0;
    c->has_state = true;
    c->ll_fresh = false;
    return MLDA_OK;
}

int mlda_set_assignments(mlda_ctx* c, const uint16_t* z, int32_t iter) {
    if (!c) return fail(MLDA_EINVAL, "null context");
    if (c->T > 0 && !z) return fail(MLDA_EINVAL, "z is null");
    if (iter < 0) return fail(MLDA_EINVAL, "iter must be >= 0");
    for (int64_t t = 0; t < c->T; ++t)
        if (z[t] >= c->K) return fail(MLDA_EINVAL, "topic >= K in z");
    if (c->T > 0) {
        uint16_t* tmp = c->z[c->cur ^ 1];
        HIP_TRY(hipMemcpyAsync(tmp, z, (size_t)c->T * 2, hipMemcpyHostToDevice, c->stream));
        hipLaunchKernelGGL(mlda::to_word_major_kernel, dim3(blocks_for(c->T, 256)), dim3(256), 0,
                           c->stream, tmp, c->tok_id, c->z[c->cur], c->T);
        HIP_TRY(hipStreamSynchronize(c->stream));     // the caller's z may go away after return
    }
    int rc = rebuild_counts(c, c->z[c->cur], nullptr, nullptr);
    if (rc != MLDA_OK) return rc;
    c->iter = iter;
    c->has_state = true;
    c->ll_fresh = false;
    return MLDA_OK;
}

int mlda_step(mlda_ctx* c, int32_t n_iters, uint32_t flags) {
    int rc = need_state(c);
    if (rc != MLDA_OK) return rc;
    if (n_iters < 0) return fail(MLDA_EINVAL, "n_iters must be >= 0");
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
        if (c->n_tiles > 0) {
            mlda::SampleArgs a;
            a.tiles = c->tiles;
            a.tok_slot = c->tok_slot;
            a.tok_id = c->tok_id;
            a.z_cur = c->z[c->cur];
            a.z_next = z_next;
            a.slots = c->slots;
            a.n_wk = c->n_wk;
            a.n_k = c->n_k;
            a.K = c->K;
            a.Kpad = c->Kpad;
            a.alpha = c->alpha;
            a.beta = c->beta;
            a.beta_V = c->beta * (double)c->V;
            a.seed = c->seed;
            a.iter = (uint32_t)(c->iter + 1);
            const int waves = sample_waves_for(c->K);
            void* kernel_args[] = {&a};
            HIP_TRY(hipLaunchKernel(sample_kernel_for(c->K, c->packed), dim3((unsigned)c->n_tiles),
                                    dim3((unsigned)(waves * mlda::kWave)), kernel_args, c->sample_lds,
                                    c->stream));
            rc = launch_check("sample_kernel");
            if (rc != MLDA_OK) return rc;
        }
        if (ev) HIP_TRY(hipEventRecord(ev[1], c->stream));
        rc = rebuild_counts(c, z_next, ev ? &ev[2] : nullptr, ev ? &ev[3] : nullptr);
        if (rc != MLDA_OK) return rc;
        c->cur ^= 1;
        c->iter += 1;
        c->ll_fresh = false;
        if (flags & MLDA_STEP_LOGLIK) {
            rc = launch_loglik(c);
            if (rc != MLDA_OK) return rc;
        }
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
    int rc = need_state(c);
    if (rc != MLDA_OK) return rc;
    if (c->T == 0) return MLDA_OK;
    if (!z) return fail(MLDA_EINVAL, "z is null");
    uint16_t* tmp = c->z[c->cur ^ 1];      // free between steps
    hipLaunchKernelGGL(mlda::to_doc_major_kernel, dim3(blocks_for(c->T, 256)), dim3(256), 0, c->stream,
                       c->z[c->cur], c->doc_map, tmp, c->T);
    HIP_TRY(hipMemcpyAsync(z, tmp, (size_t)c->T * 2, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return MLDA_OK;
}

int mlda_get_word_topic(mlda_ctx* c, int32_t* n_wk) {
    int rc = need_state(c);
    if (rc != MLDA_OK) return rc;
    if (!n_wk) return fail(MLDA_EINVAL, "n_wk is null");
    HIP_TRY(hipMemcpyAsync(n_wk, c->n_wk, (size_t)c->V * c->K * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return MLDA_OK;
}

int mlda_get_topic_totals(mlda_ctx* c, int32_t* n_k) {
    int rc = need_state(c);
    if (rc != MLDA_OK) return rc;
    if (!n_k) return fail(MLDA_EINVAL, "n_k is null");
    HIP_TRY(hipMemcpyAsync(n_k, c->n_k, (size_t)c->K * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return MLDA_OK;
}

static int fetch_row_rec(mlda_ctx* c, std::vector<uint2>& rec) {
    try { rec.resize((size_t)c->D); } catch (const std::bad_alloc&) {
        return fail(MLDA_ENOMEM, "out of host memory");
    }
    if (c->D > 0)
        HIP_TRY(hipMemcpyAsync(rec.data(), c->row_rec, (size_t)c->D * 8, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return MLDA_OK;
}

int mlda_get_doc_topic_nnz(mlda_ctx* c, int64_t* nnz) {
    int rc = need_state(c);
    if (rc != MLDA_OK) return rc;
    if (!nnz) return fail(MLDA_EINVAL, "nnz is null");
    std::vector<uint2> rec;
    rc = fetch_row_rec(c, rec);
    if (rc != MLDA_OK) return rc;
    int64_t n = 0;
    for (const uint2& r : rec) n += r.y;
    *nnz = n;
    return MLDA_OK;
}

int mlda_get_doc_topic_csr(mlda_ctx* c, int64_t* row_ptr, uint16_t* topics, int32_t* counts) {
    int rc = need_state(c);
    if (rc != MLDA_OK) return rc;
    if (!row_ptr) return fail(MLDA_EINVAL, "row_ptr is null");
    std::vector<uint2> rec;
    rc = fetch_row_rec(c, rec);
    if (rc != MLDA_OK) return rc;
    std::vector<unsigned char> slots;
    try { slots.resize(c->slots_bytes); } catch (const std::bad_alloc&) {
        return fail(MLDA_ENOMEM, "out of host memory");
    }
    if (c->slots_bytes > 0)
        HIP_TRY(hipMemcpy(slots.data(), c->slots, c->slots_bytes, hipMemcpyDeviceToHost));
    row_ptr[0] = 0;
    for (int64_t d = 0; d < c->D; ++d) row_ptr[d + 1] = row_ptr[d] + rec[d].y;
    if (row_ptr[c->D] > 0 && (!topics || !counts)) return fail(MLDA_EINVAL, "topics or counts is null");
    for (int64_t d = 0; d < c->D; ++d) {
        const uint32_t nnz = rec[d].y, pad = (nnz + 3u) & ~3u;
        const unsigned char* base = slots.data() + (size_t)rec[d].x * 16 + mlda::kRowHeader;
        if (nnz == 0) continue;
        if (c->packed) {
            const uint32_t* ent = reinterpret_cast<const uint32_t*>(base);
            for (uint32_t j = 0; j < nnz; ++j) {
                counts[row_ptr[d] + j] = (int32_t)(ent[j] >> 18);
                topics[row_ptr[d] + j] = (uint16_t)((ent[j] >> 2) & 0xffffu);
            }
        } else {
            std::memcpy(counts + row_ptr[d], base, (size_t)nnz * 4);
            std::memcpy(topics + row_ptr[d], base + (size_t)pad * 4, (size_t)nnz * 2);
        }
    }
    return MLDA_OK;
}

int mlda_get_loglik(mlda_ctx* c, double* ll) {
    int rc = need_state(c);
    if (rc != MLDA_OK) return rc;
    if (!ll) return fail(MLDA_EINVAL, "ll is null");
    if (!c->ll_fresh) {
        rc = launch_loglik(c);
        if (rc != MLDA_OK) return rc;
    }
    HIP_TRY(hipMemcpyAsync(ll, c->ll_value, 8, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return MLDA_OK;
}

int mlda_get_timing(mlda_ctx* c, double* ms, int32_t capacity_iters, int32_t* n_iters) {
    if (!c || !ms || !n_iters || capacity_iters < 0) return fail(MLDA_EINVAL, "bad argument");
    HIP_TRY(hipStreamSynchronize(c->stream));
    const int32_t n = std::min(c->timed_iters, capacity_iters);
    const int32_t first = c->timed_iters - n;
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
    int rc = need_state(c);
    if (rc != MLDA_OK) return rc;
    if (!bytes || !n_iters || capacity_iters < 0) return fail(MLDA_EINVAL, "bad argument");
    const int32_t n = std::min({c->last_step_iters, capacity_iters, kMaxTimedIters});
    // iteration j of the step (0-based, of last_step_iters) sampled from the state left by
    // rebuild number (rebuilds - last_step_iters + j - 1)
    std::vector<unsigned long long> ring((size_t)kEntryRing);
    HIP_TRY(hipMemcpyAsync(ring.data(), c->row_entries, (size_t)kEntryRing * 8, hipMemcpyDeviceToHost,
                           c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    for (int32_t i = 0; i < n; ++i) {
        const int32_t j = c->last_step_iters - n + i;
        const int64_t r = c->rebuilds - c->last_step_iters + j - 1;
        const double row_entries = c->D > 0 ? (double)ring[(size_t)(r % kEntryRing)] : 0.0;
        // per token: row slot 4, token id 4, old topic 2, new topic 2, row length 4
        bytes[i] = 16.0 * (double)c->T + (c->packed ? 4.0 : 6.0) * row_entries +
                   4.0 * (double)c->K * (double)c->n_tiles;
    }
    *n_iters = n;
    return MLDA_OK;
}

void mlda_destroy(mlda_ctx* c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    for (hipEvent_t ev : c->events) (void)hipEventDestroy(ev);
    delete c;
}

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
