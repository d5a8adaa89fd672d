// Model update kernels (paper Section 6.2): phi and n_k from the word-sorted
// assignments, theta rows from the document->token map; plus the order changes at
// the boundary and the log-likelihood reductions.
#pragma once
#include "device_util.hpp"
#include "kernels_sample.hpp"

namespace mlda {

__global__ void zero_u64_kernel(unsigned long long* p) { *p = 0ull; }

__global__ void fill_i32_kernel(int32_t* p, int64_t n, int32_t v) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// Rows of words whose tokens span several segments are accumulated with atomics and must
// start at zero.  grid = (#split words, ceil(K / blockDim)).
__global__ void zero_rows_kernel(const int32_t* words, PhiView phi, int32_t K) {
    const int k = (int)(blockIdx.y * blockDim.x + threadIdx.x);
    if (k >= K) return;
    const int v = words[blockIdx.x], wide_row = phi.wide_row[v];
    if (wide_row >= 0) phi.wide[(size_t)wide_row * (size_t)K + k] = 0;
    else phi.narrow[(size_t)v * (size_t)K + k] = 0;
}

// Update phi (Section 6.2: word by word, atomics with good locality): a workgroup
// histograms one segment (up to 16384 consecutive tokens of one word) in LDS, then stores
// the word's row outright if the segment is the whole word, else adds its non-zero bins
// to the row.  A 16-bit cell is added to through the aligned dword that holds it: the word has
// fewer than 2^16 tokens, so no sum carries into the neighbouring cell.
// kRange: K counters do not fit a workgroup's LDS; the launch then covers the topics
// k_lo .. k_lo + kn - 1 only (one launch per such range), else all K.
template <bool kRange>
__global__ __launch_bounds__(256) void phi_tile_kernel(const Tile* segs, const uint16_t* z,
                                                       PhiView phi, int32_t K, int32_t k_lo, int32_t kn) {
    extern __shared__ __align__(16) unsigned char lds[];
    int32_t* hist = reinterpret_cast<int32_t*>(lds);
    const Tile tl = segs[blockIdx.x];
    const int tid = (int)threadIdx.x;
    const int lo = kRange ? k_lo : 0, n = kRange ? kn : K;
    for (int k = tid; k < n; k += 256) hist[k] = 0;
    __syncthreads();
    // four independent loads in flight per thread: the loop is bound by their latency
    const uint16_t* zt = z + tl.begin;
    int i = tid;
    if (kRange) {
        for (; i < tl.count; i += 256) {
            const int k = (int)zt[i] - lo;
            if ((unsigned)k < (unsigned)n) atomicAdd(&hist[k], 1);
        }
    } else {
        for (; i + 768 < tl.count; i += 1024) {
            const int k0 = zt[i], k1 = zt[i + 256], k2 = zt[i + 512], k3 = zt[i + 768];
            atomicAdd(&hist[k0], 1); atomicAdd(&hist[k1], 1); atomicAdd(&hist[k2], 1); atomicAdd(&hist[k3], 1);
        }
        for (; i < tl.count; i += 256) atomicAdd(&hist[zt[i]], 1);
    }
    __syncthreads();
    const int wide_row = phi.wide_row[tl.word];
    if (wide_row >= 0) {
        int32_t* row = phi.wide + (size_t)wide_row * (size_t)K + lo;
        if (tl.whole) {
            for (int k = tid; k < n; k += 256) row[k] = hist[k];
        } else {
            for (int k = tid; k < n; k += 256) {
                const int c = hist[k];
                if (c != 0) atomicAdd(&row[k], c);
            }
        }
    } else {
        const size_t cell0 = (size_t)tl.word * (size_t)K + (size_t)lo;
        if (tl.whole) {
            for (int k = tid; k < n; k += 256) phi.narrow[cell0 + k] = (uint16_t)hist[k];
        } else {
            uint32_t* dwords = reinterpret_cast<uint32_t*>(phi.narrow);
            for (int k = tid; k < n; k += 256) {
                const uint32_t c = (uint32_t)hist[k];
                const size_t cell = cell0 + k;
                if (c != 0) atomicAdd(&dwords[cell >> 1], c << ((cell & 1) * 16));
            }
        }
    }
}

// n_k[k] = number of tokens with topic k.  Persistent workgroups, each over a contiguous
// share of the tokens; n_k must be zero on entry.  kRange as above.
template <bool kRange>
__global__ __launch_bounds__(256) void topic_totals_kernel(const uint16_t* z, int64_t T, int32_t* n_k,
                                                           int32_t K, int32_t k_lo, int32_t kn) {
    extern __shared__ __align__(16) unsigned char lds[];
    int32_t* hist = reinterpret_cast<int32_t*>(lds);
    const int tid = (int)threadIdx.x;
    const int lo = kRange ? k_lo : 0, n = kRange ? kn : K;
    for (int k = tid; k < n; k += 256) hist[k] = 0;
    __syncthreads();
    const int64_t per = (T + gridDim.x - 1) / gridDim.x;
    const int64_t t_lo = per * blockIdx.x, t_hi = (t_lo + per < T) ? t_lo + per : T;
    for (int64_t t = t_lo + tid; t < t_hi; t += 256) {
        const int k = (int)z[t] - lo;
        if (!kRange || (unsigned)k < (unsigned)n) atomicAdd(&hist[k], 1);
    }
    __syncthreads();
    for (int k = tid; k < n; k += 256) {
        const int c = hist[k];
        if (c != 0) atomicAdd(&n_k[lo + k], c);
    }
}

// The same totals as column sums of n_wk (cheaper than a pass over z when V K is small next to
// T): thread x of a workgroup owns topic blockIdx.x * 256 + x, workgroup row blockIdx.y a
// slice of the words, and the same slice of the wide rows (there are at most V of them); reads
// are coalesced along a word's row.  n_k must be zero on entry.
__global__ __launch_bounds__(256) void topic_totals_from_rows_kernel(PhiView phi, int32_t V, int32_t n_wide,
                                                                     int32_t K, int32_t words_per_slice,
                                                                     int32_t* n_k) {
    const int k = (int)(blockIdx.x * 256 + threadIdx.x);
    if (k >= K) return;
    const int v0 = (int)blockIdx.y * words_per_slice;
    int acc = 0;
    for (int v = v0; v < min(v0 + words_per_slice, V); ++v) acc += (int)phi.narrow[(size_t)v * (size_t)K + k];
    for (int r = v0; r < min(v0 + words_per_slice, n_wide); ++r) acc += phi.wide[(size_t)r * (size_t)K + k];
    if (acc != 0) atomicAdd(&n_k[k], acc);
}

// ------------------------------------------------------------------ log-likelihood helpers
// log p(w,z) = sum_k [lgG(V beta) - lgG(n_k + V beta)] + sum_{v,k} [lgG(n_wk + beta) - lgG(beta)]
//            + sum_d [lgG(K alpha) - lgG(N_d + K alpha)] + sum_{d,k} [lgG(n_dk + alpha) - lgG(alpha)]
// Each workgroup writes one fp64 partial; a last single-workgroup kernel adds them in a
// fixed order, so the value does not depend on scheduling.

__device__ __forceinline__ void block_partial_store(double v, double* partial) {
    __shared__ double wsum[16];
    const int lane = lane_id(), wave = (int)threadIdx.x / kWave;
    const double s = wave_sum(v);
    if (lane == 0) wsum[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot = 0.0;
        for (int w = 0; w < (int)blockDim.x / kWave; ++w) tot += wsum[w];
        partial[blockIdx.x] = tot;
    }
}

// lgG(c + a) - lgG(a) for the small integer counts c < kLgTable that make up almost all
// cells comes from a table, filled once per context in global memory (kLgTable entries, then
// lgG(a) itself): the kernels that use it call no lgamma and stay register-lean.
constexpr int kLgTable = 1024;

__global__ void lg_table_kernel(double* table, double a) {
    const double lg_a = lgamma(a);
    const int c = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (c < kLgTable) table[c] = lgamma((double)c + a) - lg_a;
    if (c == kLgTable) table[c] = lg_a;
}

// lgG(x) for x >= 1024 by Stirling's series; the first omitted term is below 1e-24.
__device__ __forceinline__ double lgamma_large(double x) {
    const double r = 1.0 / x, r2 = r * r;
    return (x - 0.5) * log(x) - x + 0.91893853320467274178 +
           r * (1.0 / 12.0 - r2 * (1.0 / 360.0 - r2 * (1.0 / 1260.0)));
}

// Counts of a theta row are small: the rebuild keeps only this many table entries in LDS
// (occupancy matters more there) and reads the rest of the table from global memory.
constexpr int kThetaLgTable = 128;
constexpr int kXcds = 8;            // accelerator dies of an MI355X, each with its own L2

// One document as the theta rebuild needs it, stored in processing order.
struct __align__(16) DocRec {
    int32_t begin;      // first document-major token
    int32_t n;          // tokens
    uint32_t slot;      // offset of the theta row's slot, 16-byte units
    int32_t doc;        // document id
};

// Where the topic of the document's token `j` is found in z, or -1 past the document's end:
// its word-major position, through the map; or, without a map (z in document order), the
// token's own index.
__device__ __forceinline__ int doc_token_position(const int32_t* doc_map, const DocRec& r, int j) {
    if (j >= r.n) return -1;
    return doc_map ? doc_map[r.begin + j] : r.begin + j;
}

// The same as loads that every lane makes, from an address that exists: past the document's
// end it is the place of the document's last token (of token 0 of the whole array for an empty
// document).  The loads of a step are then all in flight together and none of them sits
// behind a branch, where what follows would wait for everything in flight.
__device__ __forceinline__ int doc_token_position_any(const int32_t* doc_map, const DocRec& r, int j) {
    const int at = r.n > 0 ? r.begin + min(j, r.n - 1) : 0;
    return doc_map ? doc_map[at] : at;
}
// The topic found at such a position, -1 for a token past the document's end.
__device__ __forceinline__ int doc_token_topic(const uint16_t* z, int position, const DocRec& r, int j) {
    const int k = (int)z[position];
    return j < r.n ? k : -1;
}

// LDS bytes of the rebuild's dense row: the counters (two 16-bit counters per dword, or one
// 32-bit counter per topic when some document has 2^16 tokens or more), then one bit per topic
// that marks the non-zero bins.
// (32-bit counters for more than kThetaWideSpan topics would not fit the LDS: such a document is
// counted once per range of that many topics, and its row grows range by range.)
constexpr int32_t kThetaWideSpan = 32768;
__host__ __device__ inline int32_t theta_span(int32_t K, bool wide) {
    return wide && K > kThetaWideSpan ? kThetaWideSpan : K;
}
__host__ __device__ inline size_t theta_counter_bytes(int32_t K, bool wide) {
    const size_t counters = wide ? (size_t)theta_span(K, wide) * 4 : (size_t)((K + 1) / 2) * 4;
    return (counters + 15) & ~(size_t)15;
}
__host__ __device__ inline size_t theta_hist_bytes(int32_t K, bool wide) {
    const size_t marks = (size_t)((theta_span(K, wide) + 31) / 32) * 4;
    return theta_counter_bytes(K, wide) + ((marks + 15) & ~(size_t)15);
}
__host__ __device__ inline size_t theta_lds_bytes(int32_t K, bool wide) {
    return theta_hist_bytes(K, wide) + (size_t)kThetaLgTable * 8;
}

// Entries a count of c > 0 takes in a row whose entries hold at most kMax each.
template <class Layout>
__device__ __forceinline__ int entries_of(int c) {
    return (c + Layout::kMaxCount - 1) / Layout::kMaxCount;
}

// The entries of topic k with count c > 0, written from ent[at] on; returns the next place.
template <class Layout>
__device__ __forceinline__ int write_entries(typename Layout::Entry* ent, int at, int k, int c) {
    while (c > Layout::kMaxCount) {
        ent[at++] = Layout::make(Layout::kMaxCount, k);
        c -= Layout::kMaxCount;
    }
    ent[at++] = Layout::make(c, k);
    return at;
}

// What closes a row: padding entries up to a whole unit (lanes 0 .. 6 of `hl`), the number of
// entries at the head of the slot and a padding entry at the header's very end, so that the
// entry "before the first" is never anybody's topic.
template <class Layout>
__device__ __forceinline__ void close_row(unsigned char* head, int n_entries, int K, int hl, bool real) {
    typedef typename Layout::Entry Entry;
    Entry* ent = reinterpret_cast<Entry*>(head + kRowHeader);
    const int padded = (n_entries + Layout::kUnitEntries - 1) / Layout::kUnitEntries * Layout::kUnitEntries;
    if (real && hl < padded - n_entries) ent[n_entries + hl] = Layout::make(0, K);
    if (real && hl == 0) {
        *reinterpret_cast<uint32_t*>(head) = (uint32_t)n_entries;
        ent[-1] = Layout::make(0, K);
    }
}

// Update theta (Section 6.2): document by document, (1) a dense K-long histogram of the
// document's assignments, reached through the document->token map, (2) compaction of the
// non-zero bins into the row (topics ascending).  One wave per document, persistent; the
// dense row lives in LDS and is left all-zero for the next document.  Documents are taken in
// the order the tokens have inside a word (falling length), so that documents in flight
// together gather from neighbouring lines of z.  The walk is a chain of dependent loads
// (record -> map -> z), so it is software-pipelined: while the current document is counted,
// the topics of the wave's next document, the map entries of the one after and the record
// after that are already on their way.  Rows are written in the layout the sampler reads
// (PackedRows or TinyRows, see kernels_sample.hpp).  The compaction visits only the 32-topic
// groups that hold a non-zero bin (one mark bit per topic), so its cost follows the row's
// length rather than K.  While the counts pass through registers the kernel also adds up the
// theta entries' term of the log-likelihood, sum_{d,k} lgG(n_dk + alpha) - lgG(alpha), one
// partial per workgroup.
template <class Layout, bool kWide>
__global__ __launch_bounds__(kWave) void theta_rows_kernel(const DocRec* docs,
                                                           const int32_t* doc_map,
                                                           const uint16_t* z, uint2* row_rec,
                                                           unsigned char* slots, int64_t D, int64_t T,
                                                           int32_t K, double alpha,
                                                           const double* lg_table,
                                                           unsigned long long* row_entries,
                                                           double* ll_partial) {
    typedef typename Layout::Entry Entry;
    if (T == 0) {       // no token anywhere: the loads "past a document's end" still need a place that exists
        doc_map = nullptr;
        z = reinterpret_cast<const uint16_t*>(docs);
    }
    extern __shared__ __align__(16) unsigned char lds[];
    uint32_t* hist = reinterpret_cast<uint32_t*>(lds);
    const int span = theta_span(K, kWide);       // topics counted at a time: all, but for kWide and a very large K
    const int n_counters = kWide ? span : (K + 1) / 2;
    const int n_marks = (span + 31) / 32;
    uint32_t* marks = reinterpret_cast<uint32_t*>(lds + theta_counter_bytes(K, kWide));
    double* table = reinterpret_cast<double*>(lds + theta_hist_bytes(K, kWide));
    const int lane = (int)threadIdx.x;
    const double lg_alpha = lg_table[kLgTable];
    for (int k = lane; k < n_counters; k += kWave) hist[k] = 0u;
    for (int k = lane; k < n_marks; k += kWave) marks[k] = 0u;
    for (int c = lane; c < kThetaLgTable; c += kWave) table[c] = lg_table[c];
    __syncthreads();
    unsigned long long visited = 0;      // sum of N_d * (entries of row d) over this wave's documents
    double ll = 0.0;
    // lgG(c + alpha) - lgG(alpha) added to `ll`; the rare large counts go through a branch the
    // whole wave takes or skips, so that the common case never pays for the logarithm
    auto add_ll = [&](int c) {
        if (c > 0 && c < kThetaLgTable) ll += table[c];
        if (__ballot(c >= kThetaLgTable) != 0) {
            if (c >= kThetaLgTable)
                ll += c < kLgTable ? lg_table[c] : lgamma_large((double)c + alpha) - lg_alpha;
        }
    };
    // one more token of topic k; true if the topic's count has outgrown one entry
    auto count_topic = [&](int k) -> bool {
        atomicOr(&marks[k >> 5], 1u << (k & 31));
        if (kWide) return (int)atomicAdd(&hist[k], 1u) >= Layout::kMaxCount;
        const uint32_t before = atomicAdd(&hist[k >> 1], 1u << ((k & 1) << 4));
        return (int)((before >> ((k & 1) << 4)) & 0xffffu) >= Layout::kMaxCount;
    };
    // the same for a document too short for that (the atomics then return nothing)
    auto count_topic_short = [&](int k) {
        atomicOr(&marks[k >> 5], 1u << (k & 31));
        if (kWide) atomicAdd(&hist[k], 1u);
        else atomicAdd(&hist[k >> 1], 1u << ((k & 1) << 4));
    };
    auto count_of = [&](int k) -> int {    // (narrow counters: the pair's other half stays)
        return kWide ? (int)hist[k] : (int)((hist[k >> 1] >> ((k & 1) << 4)) & 0xffffu);
    };
    const int64_t step = gridDim.x;
    const DocRec none = {0, 0, 0u, 0};
    // workgroups are dealt to the 8 XCDs round-robin: give each XCD a contiguous run of
    // documents, so that neighbouring gathers meet in the same L2
    const int per_xcd = (int)gridDim.x / kXcds;
    int64_t i = (int)blockIdx.x < per_xcd * kXcds
                    ? (int64_t)((int)blockIdx.x % kXcds) * per_xcd + (int)blockIdx.x / kXcds
                    : (int64_t)blockIdx.x;
    // Three loads deep: the topics of this document's first 128 tokens have been gathered, the
    // positions of the next document's tokens read, and the record after that fetched.
    auto record = [&](int64_t d) {      // (the load is made for every d, from the last record if need be)
        const DocRec r = docs[d < D ? d : D - 1];
        return d < D ? r : none;
    };
    DocRec cur = record(i), nxt = record(i + step), after = record(i + 2 * step);
    int k0, k1;
    {
        const int c0 = doc_token_position_any(doc_map, cur, lane);
        const int c1 = doc_token_position_any(doc_map, cur, lane + kWave);
        k0 = doc_token_topic(z, c0, cur, lane);
        k1 = doc_token_topic(z, c1, cur, lane + kWave);
    }
    int p0 = doc_token_position_any(doc_map, nxt, lane);
    int p1 = doc_token_position_any(doc_map, nxt, lane + kWave);
    for (; i < D; i += step) {
        // on their way while this document is counted: the next document's topics, the
        // positions of the one after, the record after that
        const int n0 = doc_token_topic(z, p0, nxt, lane);
        const int n1 = doc_token_topic(z, p1, nxt, lane + kWave);
        const int q0 = doc_token_position_any(doc_map, after, lane);
        const int q1 = doc_token_position_any(doc_map, after, lane + kWave);
        const DocRec later = record(i + 3 * step);

        const bool long_doc = cur.n > Layout::kMaxCount;     // (the same for the whole wave)
        unsigned char* head = slots + (size_t)cur.slot * 16u;
        Entry* ent = reinterpret_cast<Entry*>(head + kRowHeader);
        int filled = 0, distinct = 0;
        bool any_split = false;
        // (one round, but for 32-bit counters and more topics than they have room for)
        for (int k_lo = 0; k_lo < K; k_lo += span) {
        bool outgrown = false;
        auto count = [&](int k) {
            if (k < 0) return;
            if (kWide) {
                k -= k_lo;
                if ((unsigned)k >= (unsigned)span) return;
            }
            if (long_doc) outgrown |= count_topic(k); else count_topic_short(k);
        };
        count(k0);
        count(k1);
        // the rest of a longer document, four tokens per lane at a time: their positions
        // first, then their topics, each group of loads in flight together
        for (int j = 2 * kWave + lane; j - lane < cur.n; j += 4 * kWave) {
            int at[4], k[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) at[t] = doc_token_position_any(doc_map, cur, j + t * kWave);
#pragma unroll
            for (int t = 0; t < 4; ++t) k[t] = doc_token_topic(z, at[t], cur, j + t * kWave);
#pragma unroll
            for (int t = 0; t < 4; ++t) count(k[t]);
        }
        __syncthreads();
        // some count of the document takes several entries
        const bool may_split = __ballot(outgrown) != 0;
        any_split |= may_split;
        // Each lane owns one word of marks (32 topics) per round and writes its non-zero bins
        // in ascending order behind those of the lanes below it.
        for (int base = 0; base < n_marks; base += kWave) {
            const int wi = base + lane;
            uint32_t w = wi < n_marks ? marks[wi] : 0u;
            if (__ballot(w != 0u) == 0) continue;
            int mine = __popc(w);
            distinct += mine;
            if (may_split) {           // the lane's entries, counted one bin at a time
                mine = 0;
                for (uint32_t rest = w; rest != 0u; rest &= rest - 1u)
                    mine += entries_of<Layout>(count_of(wi * 32 + __ffs((int)rest) - 1));
            }
            const int upto = wave_inclusive_sum(mine);
            int at = filled + upto - mine;
            filled += read_lane(upto, kWave - 1);
            if (w != 0u) marks[wi] = 0u;
            if (kWide) {
                while (__ballot(w != 0u) != 0) {
                    int c = 0;
                    if (w != 0u) {
                        const int k = wi * 32 + __ffs((int)w) - 1;
                        w &= w - 1u;
                        c = (int)hist[k];
                        hist[k] = 0u;
                        at = write_entries<Layout>(ent, at, k_lo + k, c);
                    }
                    add_ll(c);
                }
            } else {
                uint32_t pairs = (w | (w >> 1)) & 0x55555555u;
                while (__ballot(pairs != 0u) != 0) {
                    int lo = 0, hi = 0;
                    if (pairs != 0u) {
                        const int k = wi * 32 + __ffs((int)pairs) - 1;    // even topic of the pair
                        pairs &= pairs - 1u;
                        const uint32_t both = hist[k >> 1];
                        hist[k >> 1] = 0u;
                        lo = (int)(both & 0xffffu);
                        hi = (int)(both >> 16);
                        if (lo != 0) at = write_entries<Layout>(ent, at, k, lo);
                        if (hi != 0) at = write_entries<Layout>(ent, at, k + 1, hi);
                    }
                    add_ll(lo);
                    add_ll(hi);
                }
            }
        }
        if (k_lo + span < K) __syncthreads();
        }
        close_row<Layout>(head, filled, K, lane, true);
        const int nnz = any_split ? wave_sum(distinct) : filled;
        if (lane == 0) row_rec[cur.doc].y = (uint32_t)nnz;      // distinct topics, for the getters
        visited += (unsigned long long)cur.n * (unsigned long long)filled;
        __syncthreads();
        cur = nxt; nxt = after; after = later; k0 = n0; k1 = n1; p0 = q0; p1 = q1;
    }
    // row entries the next sampling pass will read: one row walk per token
    if (lane == 0 && visited != 0) atomicAdd(row_entries, visited);
    block_partial_store(ll, ll_partial);
}

// The same for K <= 1024 and documents of fewer than 2^16 tokens, two documents per wave: the
// mark bits of a document then fit one word per lane of a half-wave (32 lanes x 32 topics), so
// lanes 0..31 rebuild one document and lanes 32..63 the next one with the same instructions,
// which halves the instructions per document.  Documents 2 p and 2 p + 1 (neighbours in the
// working order, so of similar length) make pair p; the topics of the first 128 tokens of each
// document of the next pair are on their way while the current pair is counted.
constexpr int kPairMaxK = 1024;
constexpr int kPairStage = 256;         // entries of a row that are lined up in LDS before they are stored
__host__ __device__ inline size_t theta_pair_lds_bytes(int32_t K) {
    return 2 * theta_hist_bytes(K, false) + (size_t)kThetaLgTable * 8 + 2 * (size_t)kPairStage * 4;
}

template <class Layout>
__global__ __launch_bounds__(kWave) void theta_rows_pair_kernel(const DocRec* docs,
                                                                const int32_t* doc_map,
                                                                const uint16_t* z, uint2* row_rec,
                                                                unsigned char* slots, int64_t D, int64_t T,
                                                                int32_t K, double alpha,
                                                                const double* lg_table,
                                                                unsigned long long* row_entries,
                                                                double* ll_partial) {
    typedef typename Layout::Entry Entry;
    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = (int)threadIdx.x, half = lane >> 5, hl = lane & 31;
    const int n_counters = (K + 1) / 2, n_marks = (K + 31) / 32;
    const size_t one = theta_hist_bytes(K, false);
    // per half: paired 16-bit counters, then one mark bit per topic
    uint32_t* hist = reinterpret_cast<uint32_t*>(lds + (size_t)half * one);
    uint32_t* marks = reinterpret_cast<uint32_t*>(lds + (size_t)half * one + theta_counter_bytes(K, false));
    double* table = reinterpret_cast<double*>(lds + 2 * one);
    // per half: room to line up a row's entries before they are stored
    Entry* stage = reinterpret_cast<Entry*>(lds + 2 * one + (size_t)kThetaLgTable * 8) + half * kPairStage;
    const double lg_alpha = lg_table[kLgTable];
    for (int k = hl; k < n_counters; k += 32) hist[k] = 0u;
    for (int k = hl; k < n_marks; k += 32) marks[k] = 0u;
    for (int c = lane; c < kThetaLgTable; c += kWave) table[c] = lg_table[c];
    __syncthreads();
    unsigned long long visited = 0;      // sum of N_d * (entries of row d) over this half's documents
    double ll = 0.0;
    auto add_ll = [&](int c) {
        if (c > 0 && c < kThetaLgTable) ll += table[c];
        if (__ballot(c >= kThetaLgTable) != 0) {
            if (c >= kThetaLgTable)
                ll += c < kLgTable ? lg_table[c] : lgamma_large((double)c + alpha) - lg_alpha;
        }
    };
    // one more token of topic k; true if the topic's count has outgrown one entry
    auto count_topic = [&](int k) -> bool {
        const uint32_t before = atomicAdd(&hist[k >> 1], 1u << ((k & 1) << 4));
        atomicOr(&marks[k >> 5], 1u << (k & 31));
        return (int)((before >> ((k & 1) << 4)) & 0xffffu) >= Layout::kMaxCount;
    };
    auto topic_at = [&](const DocRec& r, int j) {       // topic of the document's token j, -1 past its end
        const int p = doc_token_position(doc_map, r, j);
        return p >= 0 ? (int)z[p] : -1;
    };
    const int64_t n_pairs = (D + 1) / 2, step = gridDim.x;
    const DocRec none = {0, 0, 0u, 0};
    auto record = [&](int64_t p) { return (p < n_pairs && 2 * p + half < D) ? docs[2 * p + half] : none; };
    // each XCD takes a contiguous run of pairs (see theta_rows_kernel)
    const int per_xcd = (int)gridDim.x / kXcds;
    int64_t i = (int)blockIdx.x < per_xcd * kXcds
                    ? (int64_t)((int)blockIdx.x % kXcds) * per_xcd + (int)blockIdx.x / kXcds
                    : (int64_t)blockIdx.x;
    DocRec cur = record(i), nxt = record(i + step);
    int k0 = topic_at(cur, hl), k1 = topic_at(cur, hl + 32), k2 = topic_at(cur, hl + 64),
        k3 = topic_at(cur, hl + 96);
    for (; i < n_pairs; i += step) {
        const int n0 = topic_at(nxt, hl), n1 = topic_at(nxt, hl + 32), n2 = topic_at(nxt, hl + 64),
                  n3 = topic_at(nxt, hl + 96);
        const DocRec after = record(i + 2 * step);
        bool outgrown = false;
        if (k0 >= 0) outgrown |= count_topic(k0);
        if (k1 >= 0) outgrown |= count_topic(k1);
        if (k2 >= 0) outgrown |= count_topic(k2);
        if (k3 >= 0) outgrown |= count_topic(k3);
        for (int j = 128 + hl; j < cur.n; j += 32) outgrown |= count_topic(topic_at(cur, j));
        __syncthreads();
        unsigned char* head = slots + (size_t)cur.slot * 16u;
        Entry* ent = reinterpret_cast<Entry*>(head + kRowHeader);
        // lane hl of a half owns mark word hl: 32 topics = 16 counter pairs
        const uint32_t w = hl < n_marks ? marks[hl] : 0u;
        const int distinct = __popc(w);
        int mine = distinct;
        if (__ballot(outgrown) != 0) {      // some count of the pair takes several entries
            mine = 0;
            for (uint32_t rest = w; rest != 0u; rest &= rest - 1u) {
                const int k = hl * 32 + __ffs((int)rest) - 1;
                mine += entries_of<Layout>((int)((hist[k >> 1] >> ((k & 1) << 4)) & 0xffffu));
            }
        }
        // prefix over the 32 lanes of each half: the wave-wide scan without its last step
        auto half_inclusive_sum = [](int v) {
            v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);
            v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);
            v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);
            v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);
            v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);
            return v;
        };
        const int upto = half_inclusive_sum(mine);
        const int n_a = read_lane(upto, 31), n_b = read_lane(upto, 63);
        const int n_entries = half ? n_b : n_a;
        int nnz = n_entries;                              // distinct topics of the row
        if (__ballot(mine != distinct) != 0) {
            const int d_upto = half_inclusive_sum(distinct);
            const int d_a = read_lane(d_upto, 31), d_b = read_lane(d_upto, 63);
            nnz = half ? d_b : d_a;
        }
        int at = upto - mine;
        if (w != 0u) marks[hl] = 0u;
        uint32_t pairs = (w | (w >> 1)) & 0x55555555u;
        const bool real = 2 * i + half < D;              // the last pair may lack its second document
        const int n_longer = max(n_a, n_b);
        if (__ballot(mine != distinct) == 0 && n_longer <= kPairStage) {
            // The usual case, every topic one entry: the lanes that own the bins only line the
            // entries up in LDS; the lanes then take them one each, so that the row leaves in
            // whole consecutive stores and the likelihood's term is added with all lanes busy.
            while (__ballot(pairs != 0u) != 0) {
                if (pairs != 0u) {
                    const int k = hl * 32 + __ffs((int)pairs) - 1;    // even topic of the pair
                    pairs &= pairs - 1u;
                    const uint32_t both = hist[k >> 1];
                    hist[k >> 1] = 0u;
                    const int lo = (int)(both & 0xffffu), hi = (int)(both >> 16);
                    if (lo != 0) stage[at++] = Layout::make(lo, k);
                    if (hi != 0) stage[at++] = Layout::make(hi, k + 1);
                }
            }
            __syncthreads();
            for (int first = 0; first < n_longer; first += 32) {
                const int e = first + hl;
                int c = 0;
                if (e < n_entries) {
                    const Entry v = stage[e];
                    ent[e] = v;
                    c = Layout::entry_count(v);
                }
                add_ll(c);
            }
        } else {
            while (__ballot(pairs != 0u) != 0) {
                int lo = 0, hi = 0;
                if (pairs != 0u) {
                    const int k = hl * 32 + __ffs((int)pairs) - 1;    // even topic of the pair
                    pairs &= pairs - 1u;
                    const uint32_t both = hist[k >> 1];
                    hist[k >> 1] = 0u;
                    lo = (int)(both & 0xffffu);
                    hi = (int)(both >> 16);
                    if (lo != 0) at = write_entries<Layout>(ent, at, k, lo);
                    if (hi != 0) at = write_entries<Layout>(ent, at, k + 1, hi);
                }
                add_ll(lo);
                add_ll(hi);
            }
        }
        close_row<Layout>(head, n_entries, K, hl, real);
        if (real && hl == 0) {
            row_rec[cur.doc].y = (uint32_t)nnz;          // distinct topics, for the getters
            visited += (unsigned long long)cur.n * (unsigned long long)n_entries;
        }
        __syncthreads();
        cur = nxt; nxt = after; k0 = n0; k1 = n1; k2 = n2; k3 = n3;
    }
    if (hl == 0 && visited != 0) atomicAdd(row_entries, visited);
    block_partial_store(ll, ll_partial);
}

// The two per-token index arrays that follow from tok_id and the document records are built
// on the device rather than sent over PCIe.  doc_map (Section 6.2's document->token map) is the
// inverse of tok_id; tokens are numbered from `first` inside a chunk.
__global__ void derive_doc_map_kernel(const int32_t* tok_id, int64_t T, int64_t first, int32_t* doc_map) {
    const int64_t pos = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pos < T) doc_map[(int64_t)tok_id[pos] - first] = (int32_t)pos;
}

// tok_slot[pos] = slot of the theta row of the document that owns word-major token pos.  One
// wave per document, persistent.
__global__ __launch_bounds__(kWave) void derive_tok_slot_kernel(const DocRec* docs, int64_t D,
                                                                const int32_t* doc_map,
                                                                uint32_t* tok_slot) {
    const int lane = (int)threadIdx.x;
    for (int64_t i = blockIdx.x; i < D; i += gridDim.x) {
        const DocRec r = docs[i];
        for (int j = lane; j < r.n; j += kWave) tok_slot[doc_map[r.begin + j]] = r.slot;
    }
}

// The map entries of every document put in rising order, in runs of kMapSortRun entries (a
// whole document if it has no more).  The rebuild counts a document's topics, so the order in
// which it meets them is free; in rising order the tokens that share their document AND their
// word are neighbours in the map as they are in z, neighbouring lanes then read the same line,
// and the gather asks the caches for it once.  After this the map no longer tells a token's
// place inside its document: only the rebuild and derive_tok_slot_kernel read it.
// One wave per document, persistent; a bitonic network over a run held in LDS.
constexpr int kMapSortRun = 256;
__global__ __launch_bounds__(kWave) void sort_doc_map_kernel(const DocRec* docs, int64_t D, int32_t* doc_map) {
    __shared__ int32_t run[kMapSortRun];
    const int lane = (int)threadIdx.x;
    for (int64_t i = blockIdx.x; i < D; i += gridDim.x) {
        const DocRec r = docs[i];
        for (int base = 0; base < r.n; base += kMapSortRun) {
            const int n = min(kMapSortRun, r.n - base);
            if (n < 2) continue;
            // the smallest power of two that holds the run; places past its end sort last
            int width = 2;
            while (width < n) width <<= 1;
            for (int e = lane; e < width; e += kWave)
                run[e] = e < n ? doc_map[r.begin + base + e] : 0x7fffffff;
            __syncthreads();
            for (int k = 2; k <= width; k <<= 1)
                for (int j = k >> 1; j > 0; j >>= 1) {
                    for (int pair = lane; pair < width / 2; pair += kWave) {
                        const int lo = ((pair & ~(j - 1)) << 1) | (pair & (j - 1)), hi = lo | j;
                        const int32_t a = run[lo], b = run[hi];
                        const bool rising = (lo & k) == 0;
                        if ((a > b) == rising) { run[lo] = b; run[hi] = a; }
                    }
                    __syncthreads();
                }
            for (int e = lane; e < n; e += kWave) doc_map[r.begin + base + e] = run[e];
            __syncthreads();
        }
    }
}

// A chunk without a map (its assignments arrive in document order): every token's topic is
// paired with the slot of its document's theta row, one wave per document, persistent, where
// both are contiguous ...
__global__ __launch_bounds__(kWave) void pair_topics_with_slots_kernel(const DocRec* docs, int64_t D,
                                                                       const uint16_t* z_doc, uint2* pairs) {
    const int lane = (int)threadIdx.x;
    for (int64_t i = blockIdx.x; i < D; i += gridDim.x) {
        const DocRec r = docs[i];
        for (int j = lane; j < r.n; j += kWave)
            pairs[r.begin + j] = make_uint2(r.slot, (uint32_t)z_doc[r.begin + j]);
    }
}

// ... and one gather per word-major token brings both along (tok_id counts from the start of
// the whole corpus, the pairs from token `first`).
__global__ void pairs_to_word_major_kernel(const uint2* pairs, const int32_t* tok_id, uint16_t* z_word,
                                           uint32_t* tok_slot, int64_t T, int64_t first) {
    const int64_t pos = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pos >= T) return;
    const uint2 p = pairs[(int64_t)tok_id[pos] - first];
    tok_slot[pos] = p.x;
    z_word[pos] = (uint16_t)p.y;
}

// Boundary order changes.  tok_id[pos] = document-major index of word-major position pos.
__global__ void to_doc_major_scatter_kernel(const uint16_t* z_word, const int32_t* tok_id,
                                            uint16_t* z_doc, int64_t T, int64_t first) {
    const int64_t pos = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pos < T) z_doc[(int64_t)tok_id[pos] - first] = z_word[pos];
}

// (tok_id counts from the start of the whole corpus, z_doc from token `first`: a chunk of
// documents holds the tokens first .. first + T - 1.)
__global__ void to_word_major_kernel(const uint16_t* z_doc, const int32_t* tok_id,
                                     uint16_t* z_word, int64_t T, int64_t first) {
    const int64_t pos = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pos < T) z_word[pos] = z_doc[(int64_t)tok_id[pos] - first];
}

// ------------------------------------------------------------------ log-likelihood kernels

// Word side: sum over all cells of lgG(n_wk + beta) - lgG(beta), plus the topic totals' term.
// The 16-bit cells are read eight at a time, the 32-bit cells of the wide rows four at a time
// (empty cells add nothing, so the unused 16-bit rows of the wide words do not matter); the
// table of small counts comes ready-made from global memory (lg_table: kLgTable entries, then
// lgG(beta)), larger counts use Stirling's series.
__global__ __launch_bounds__(256) void loglik_word_side_kernel(PhiView phi, int64_t n_narrow_cells,
                                                               int64_t n_wide_cells,
                                                               const int32_t* n_k, int32_t K,
                                                               double beta, double v_beta,
                                                               const double* lg_table,
                                                               double* partial) {
    __shared__ double table[kLgTable];
    for (int c = (int)threadIdx.x; c < kLgTable; c += 256) table[c] = lg_table[c];
    const double lg_beta = lg_table[kLgTable];
    __syncthreads();
    double acc = 0.0;
    auto add_cell = [&](int c) {
        if (c > 0 && c < kLgTable) acc += table[c];
        if (__ballot(c >= kLgTable) != 0) {          // rare: taken by the whole wave or not at all
            if (c >= kLgTable) acc += lgamma_large((double)c + beta) - lg_beta;
        }
    };
    auto add_pair = [&](uint32_t two) { add_cell((int)(two & 0xffffu)); add_cell((int)(two >> 16)); };
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    {
        const int64_t n_octs = n_narrow_cells / 8;
        const uint4* octs = reinterpret_cast<const uint4*>(phi.narrow);
        int64_t i = first;
        for (; i + 3 * stride < n_octs; i += 4 * stride) {     // four loads in flight per thread
            const uint4 v0 = octs[i], v1 = octs[i + stride], v2 = octs[i + 2 * stride],
                        v3 = octs[i + 3 * stride];
            if (__ballot((v0.x | v0.y | v0.z | v0.w | v1.x | v1.y | v1.z | v1.w | v2.x | v2.y | v2.z | v2.w |
                          v3.x | v3.y | v3.z | v3.w) != 0) == 0)
                continue;
            add_pair(v0.x); add_pair(v0.y); add_pair(v0.z); add_pair(v0.w);
            add_pair(v1.x); add_pair(v1.y); add_pair(v1.z); add_pair(v1.w);
            add_pair(v2.x); add_pair(v2.y); add_pair(v2.z); add_pair(v2.w);
            add_pair(v3.x); add_pair(v3.y); add_pair(v3.z); add_pair(v3.w);
        }
        for (; i < n_octs; i += stride) {
            const uint4 v = octs[i];
            if (__ballot((v.x | v.y | v.z | v.w) != 0) == 0) continue;
            add_pair(v.x); add_pair(v.y); add_pair(v.z); add_pair(v.w);
        }
    }
    {
        const int64_t n_quads = n_wide_cells / 4;
        const int4* quads = reinterpret_cast<const int4*>(phi.wide);
        for (int64_t i = first; i < n_quads; i += stride) {
            const int4 v = quads[i];
            if (__ballot((v.x | v.y | v.z | v.w) != 0) == 0) continue;
            add_cell(v.x); add_cell(v.y); add_cell(v.z); add_cell(v.w);
        }
    }
    if (blockIdx.x == 0) {
        // up to seven 16-bit cells and up to three 32-bit cells are left
        const int64_t i = n_narrow_cells / 8 * 8 + (int64_t)threadIdx.x;
        add_cell(i < n_narrow_cells ? (int)phi.narrow[i] : 0);
        const int64_t j = n_wide_cells / 4 * 4 + (int64_t)threadIdx.x;
        add_cell(j < n_wide_cells ? phi.wide[j] : 0);
        const double lg_vb = lgamma(v_beta);
        for (int k = (int)threadIdx.x; k < K; k += (int)blockDim.x)
            acc += lg_vb - lgamma((double)n_k[k] + v_beta);
    }
    block_partial_store(acc, partial);
}

// The per-document term lgG(K alpha) - lgG(N_d + K alpha), one thread per document (the
// entries of the theta rows are summed by theta_rows_kernel).
__global__ __launch_bounds__(256) void loglik_doc_term_kernel(const int32_t* doc_ptr, int64_t D,
                                                              double k_alpha, double* partial) {
    const double lg_ka = lgamma(k_alpha);
    double acc = 0.0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t d = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; d < D; d += stride)
        acc += lg_ka - lgamma((double)(doc_ptr[d + 1] - doc_ptr[d]) + k_alpha);
    block_partial_store(acc, partial);
}

// out = (add_to_out ? *out : 0) + sum of the n partials + *extra (if given).  One workgroup,
// fixed order.
__global__ __launch_bounds__(256) void loglik_final_kernel(const double* partial, int n,
                                                           const double* extra, int add_to_out,
                                                           double* out) {
    __shared__ double buf[256];
    double acc = 0.0;
    for (int i = (int)threadIdx.x; i < n; i += 256) acc += partial[i];
    if (threadIdx.x == 0) {
        if (extra) acc += *extra;
        if (add_to_out) acc += *out;
    }
    buf[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) buf[threadIdx.x] += buf[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = buf[0];
}

}  // namespace mlda
