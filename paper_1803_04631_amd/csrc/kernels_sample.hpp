// Sampling kernel: one pass of the sparsity-aware sampler (paper Section 6.1, Eq. 6-8,
// Algorithm 2) over word-sorted tokens.
//
// Mapping to gfx950 (the paper's own mapping, one 32-wide warp per sampler with 32-way
// index trees, was made for NVIDIA warps; measured here, a whole 64-lane wave per token is
// bound by VALU issue, not by HBM):
//   - a workgroup owns one tile = up to 1024 (4096 for large K) consecutive tokens of ONE
//     word and stages that word's p*(k) (Eq. 8) once in LDS as fp32, with fp64 prefix sums
//     over groups of 4 (or 16) topics (Section 6.1.2: samplers of a block share the word's data);
//     for large K, the many words of few tokens are taken in runs by one workgroup, which turns
//     p* of one word into p* of the next; where K is too large for p* to fit the LDS at all, it
//     is staged in a strip of device memory that the workgroup owns, and read from there;
//   - each wave takes 64 tokens at a time (fewer when a large-K tile is too small to give every
//     wave that many).  What is per token and needs no cooperation is
//     done one token per LANE: the Philox uniform, the token's own-count correction of
//     p*(o), and the search in the dense bucket p2 (binary search over the group prefixes,
//     then the group's topics);
//   - the walk over the token's sparse theta row (S and the p1 prefix sums, Eq. 6-7) is done
//     by a GROUP of 4, 8, 16, 32 or 64 lanes per token, chosen per pass from the row lengths
//     so that a lane owns at most three 16-byte units of entries (16, 8, 4, 2 or 1 tokens per
//     pass: the fixed cost of a pass is shared by as many tokens as their rows allow).  Groups
//     narrower than a DPP row of 16 lanes are interleaved inside the row (4 or 2 tokens side by
//     side), so that plain row shifts scan every group at once.  Every lane owns a contiguous
//     run of entries, accumulates them in fp64 and keeps the sum at the end of each unit; a DPP
//     scan over the group gives the prefix over lanes.  The lane whose range holds the draw
//     names the unit that holds it and what is left of the draw there; "the smallest k whose
//     prefix exceeds it" (Section 6.1.1) among that unit's few entries is found afterwards, one
//     token per lane again, for all tokens of the batch at once.  Rows too long for three
//     units per lane of a whole wave are walked twice by the wave.  Token parameters and
//     results travel between the per-lane and per-group phases through small per-wave LDS
//     records;
//   - a theta row is a run of entries (topic, count) in ascending topic order, 2 bytes each
//     when K < 1024 (10 bits of topic, 4 of count), else 4 bytes (16 bits of topic, 14 of
//     count); a count too large for its field is written as several entries of the same
//     topic, one after the other, which changes no sum.  Only the first entry of the token's
//     own topic gives up the token itself;
//   - the row walk is a chain of dependent loads (record, then a random row in HBM), so the
//     loads of the next pass are issued before the current pass is worked on.
#pragma once
#include <type_traits>
#include "device_util.hpp"

namespace mlda {

struct Tile {          // consecutive word-major tokens of one word
    int32_t word;
    int32_t begin;     // first word-major token position
    int32_t count;     // 1 .. tile size
    int32_t whole;     // phi segments: 1 if the segment holds every token of its word;
                       // sampling tiles: the word's row in PhiView::wide, or -1
};

// phi (Section 6.1.3: short integers for the dense model).  A word with fewer than 2^16 tokens
// can never overflow a 16-bit count: its row lives in `narrow`.  The few heavier words have an
// int32 row in `wide` (wide_row[v] = its index there, -1 for the others) and their rows in
// `narrow` stay zero, so that sums over all cells of both matrices count every token once.
constexpr int kNarrowWordLimit = 1 << 16;   // tokens of a word from which its row is wide
struct PhiView {
    uint16_t* narrow;           // [V][K]
    int32_t* wide;              // [n_wide][K]
    const int32_t* wide_row;    // [V]
};

struct SampleArgs {
    const Tile* tiles;
    const uint32_t* tok_slot;   // [T] slot of the theta row of each word-major token's document
    const int32_t* tok_id;      // [T] its index in the caller's document-major order
    const uint16_t* z_cur;      // [T] word-major, frozen for the pass
    uint16_t* z_next;           // [T] word-major, written
    // theta rows: a slot (offset in 16-byte units) starts with a header of kRowHeader bytes
    // whose first word is the row's number of entries and whose last bytes are a padding
    // entry, then holds the entries in one of the two layouts below (PackedRows / TinyRows),
    // filled up to a whole 16-byte unit with padding entries (count 0, topic K)
    const unsigned char* slots;
    PhiView phi;
    const int32_t* n_k;         // [K]
    int32_t K, Kpad;            // Kpad = K+1 rounded up to a multiple of the dense group: p*(K..Kpad-1) = 0
    double alpha, beta, beta_V;
    uint64_t seed;
    uint32_t iter;
    // Workgroup b < n_single takes tile b.  The tiles from n_single on each hold a whole word of
    // few tokens; a workgroup takes a run of run_tiles of them, one after the other, and turns
    // p* of one word into p* of the next instead of staging it afresh (run_tiles <= 1: no runs).
    int32_t n_tiles, n_single, run_tiles;
    // K too large for p* to fit a workgroup's LDS (sample_kernel<12, .., true>): workgroup b keeps
    // p* of its current tile in far_pstar[b * Kpad ..] and takes the tiles b, b + grid, ...
    float* far_pstar;
};

constexpr int kRowHeader = 16;  // bytes before a theta row's entries
// Topics per fp64 prefix group of the dense bucket: 4 where LDS has room (workgroups of four
// waves, K <= 2048), 16 for the large-K workgroups of twelve waves.
__host__ __device__ constexpr int dense_group(int waves) { return waves == 4 ? 4 : 16; }
constexpr int kKeptUnits = 3;   // 16-byte units of entries a lane keeps in registers at most
constexpr int kMinBatch = 8;    // tokens a wave takes at a time at least

// Once a token's pass has read its record, the record takes the result back to the per-lane
// phase: `nnz` says what kind (below), `off` and `u` hold it.
struct __align__(16) TokenRec { // per-lane phase -> per-group phase, 32 bytes
    uint32_t off;               // slot offset of the token's theta row, 16-byte units
    int32_t nnz;                // 16-byte units of entries of the row
    int32_t o;                  // current topic
    float w_o;                  // p*(o) with the token itself removed
    double u;
    double Qp;                  // alpha * sum_k p*'(k)
};
constexpr int kDrawInUnit = -1; // off = the 16-byte unit of the slot buffer that holds the draw,
                                // u = what is left of the draw at the unit's start
constexpr int kDrawDense = -2;  // the draw falls into the dense bucket p2; u = its position there
constexpr int kDrawTopic = -3;  // off = the new topic itself

// LDS bytes of sample_kernel<kWaves> for a given Kpad.
__host__ __device__ constexpr size_t sample_lds_bytes(int Kpad, int waves) {
    return (size_t)Kpad * 4 + (size_t)((Kpad / dense_group(waves) + 1) & ~1) * 8 +
           (size_t)waves * kWave * sizeof(TokenRec);
}
// The same when p* stays in device memory: the prefix sums and the waves' records only.
__host__ __device__ constexpr size_t sample_far_lds_bytes(int Kpad, int waves) {
    return sample_lds_bytes(Kpad, waves) - (size_t)Kpad * 4;
}
// What runs of small tiles keep in LDS besides: the groups' own sums (the prefix sums are made
// from them again after every change) and one bit per group for "changed".
__host__ __device__ constexpr size_t sample_run_lds_bytes(int Kpad, int waves) {
    const size_t ng = (size_t)(Kpad / dense_group(waves));
    return ((ng + 1) & ~(size_t)1) * 8 + ((ng + 31) / 32 * 4 + 15 & ~(size_t)15);
}
constexpr int kRunTileTokens = 1024;    // a tile of a run holds a whole word of at most this many tokens

// Dense bucket (p2 = alpha p*', Eq. 6): smallest k with alpha * prefix'(k) > y, where
// prefix' is the prefix sum of p* with the entry of the token's own topic o replaced by
// w_o (delta = w_o - p*(o)).  One lane per token.
template <int kGroup>
__device__ __forceinline__ int dense_bucket_search(const float* pstar, const double* cp, int K,
                                                   int ng, double alpha, double y, int o,
                                                   float w_o, double delta) {
    // Bisection with steps of falling powers of two: `lo` counts the groups known to lie
    // before the draw.  Every lane makes the same number of steps, so the scalar unit runs the
    // loop, and a step is one LDS read, the correction and one comparison.
    const int o_group = o / kGroup;        // groups from here on hold the own topic's correction
    int lo = 0;
    for (int step = 1 << (31 - __builtin_clz(ng)); step > 0; step >>= 1) {
        const int upto = lo + step;        // would groups 0 .. upto - 1 all lie before the draw?
        if (upto <= ng) {
            const double pre = cp[upto - 1] + (upto > o_group ? delta : 0.0);
            if (!(alpha * pre > y)) lo = upto;
        }
    }
    if (lo >= ng) return K - 1;
    const int k0 = lo * kGroup;
    const double before = (lo > 0 ? cp[lo - 1] : 0.0) + (k0 > o ? delta : 0.0);
    if (kGroup == 4) {
        // the four topics of group `lo`, taken in one read (p* beyond K is 0 and adds nothing)
        const float4 w = *reinterpret_cast<const float4*>(pstar + k0);
        const double a0 = before + (double)(k0 == o ? w_o : w.x);
        const double a1 = a0 + (double)(k0 + 1 == o ? w_o : w.y);
        const double a2 = a1 + (double)(k0 + 2 == o ? w_o : w.z);
        int found = k0 + 3;
        if (alpha * a2 > y) found = k0 + 2;
        if (alpha * a1 > y) found = k0 + 1;
        if (alpha * a0 > y) found = k0;
        return min(found, K - 1);
    }
    double acc = before;
    int found = min(k0 + kGroup - 1, K - 1);
    for (int j = 0; j < kGroup; ++j) {
        const int k = k0 + j;
        if (k >= K) break;
        acc += (double)((k == o) ? w_o : pstar[k]);
        if (alpha * acc > y) { found = k; break; }
    }
    return found;
}

// DPP move of a double with full row and bank masks; lanes without a source read 0.
template <int kCtrl>
__device__ __forceinline__ double dpp_move_all0(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), kCtrl, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), kCtrl, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

// Lane layout of a pass with kLanes lanes per token.  Groups of 16, 32 or 64 lanes are runs
// of consecutive lanes.  Groups of 8 or 4 lanes are interleaved inside each row of 16 lanes:
// with g = 16 / kLanes tokens per row, lane l of the row works for token l % g as its
// sub-lane l / g.
//
// Inclusive prefix sum over the sub-lanes of every group.  Every lane must be active.
// Shifts inside each row of 16 lanes (starting at the interleave distance); for wider groups
// lane 15 of the even rows is added to the odd rows, and for the whole wave lane 31 to rows
// 2 and 3.
template <int kLanes>
__device__ __forceinline__ double group_inclusive_sum(double v) {
    if (kLanes >= 16) v += dpp_move_all0<0x111>(v);   // row_shr:1
    if (kLanes >= 8) v += dpp_move_all0<0x112>(v);    // row_shr:2
    v += dpp_move_all0<0x114>(v);                      // row_shr:4
    v += dpp_move_all0<0x118>(v);                      // row_shr:8
    if (kLanes >= 32) v += dpp_move0<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    if (kLanes >= 64) v += dpp_move0<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}

// Value of the sub-lane before this one inside the group, 0 for the group's first sub-lane.
template <int kLanes>
__device__ __forceinline__ double group_previous(double incl, int sl) {
    if (kLanes == 16) return dpp_move_all0<0x111>(incl);          // row_shr:1
    if (kLanes == 8) return dpp_move_all0<0x112>(incl);           // row_shr:2
    if (kLanes == 4) return dpp_move_all0<0x114>(incl);           // row_shr:4
    const double up = dpp_move_all0<0x138>(incl);                  // wave_shr:1
    return sl == 0 ? 0.0 : up;
}

// Lane that holds the group's last sub-lane.
template <int kLanes>
__device__ __forceinline__ int group_last_lane(int lane) {
    return kLanes >= 16 ? (lane | (kLanes - 1)) : (lane | (16 - 16 / kLanes));
}

// Value of the sub-lane before this one inside the group (garbage for the group's first).
template <int kLanes>
__device__ __forceinline__ int group_previous_int(int v) {
    if (kLanes == 16) return __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    if (kLanes == 8) return __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);    // row_shr:2
    if (kLanes == 4) return __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);    // row_shr:4
    return __builtin_amdgcn_update_dpp(0, v, 0x138, 0xf, 0xf, true);                      // wave_shr:1
}

// ---------------------------------------------------------------- theta row layouts
// A row's entries follow its 16-byte header in ascending topic order and are read in units of
// 16 bytes.  A count beyond an entry's field is spread over several entries of the same topic.
// key = 4 * topic = the byte offset of p*(topic) in LDS.

// 4 bytes per entry: count << 18 | topic << 2.  Any K.
struct PackedRows {
    typedef uint32_t Entry;
    static constexpr int kEntryBytes = 4, kUnitEntries = 4;
    static constexpr int kMaxCount = (1 << 14) - 1;
    static constexpr int kWavesPerSimd = 6;
    static constexpr bool kOneEntryPerTopic = false;
    static __host__ __device__ __forceinline__ Entry make(int count, int topic) {
        return ((uint32_t)count << 18) | ((uint32_t)topic << 2);
    }
    static __host__ __device__ __forceinline__ int entry_topic(Entry e) { return (int)((e >> 2) & 0xffffu); }
    static __host__ __device__ __forceinline__ int entry_count(Entry e) { return (int)(e >> 18); }
    static __device__ __forceinline__ uint32_t word(const uint4& u, int j) {
        return j == 0 ? u.x : j == 1 ? u.y : j == 2 ? u.z : u.w;
    }
    static __device__ __forceinline__ int key(const uint4& u, int j) { return (int)(word(u, j) & 0x3fffcu); }
    static __device__ __forceinline__ int count(const uint4& u, int j) { return (int)(word(u, j) >> 18); }
};

// The same when no document has more tokens than an entry counts (the host checks): every topic
// then has one entry, the row walk needs no look at the entry before, and with so few entries
// per unit the search for the draw's entry is cheapest inside the pass itself.
struct PackedRowsShort : PackedRows {
    static constexpr bool kOneEntryPerTopic = true;
};

// 2 bytes per entry: count << 12 | topic << 2 (ten bits of topic, four of count).  K < 1024.
struct TinyRows {
    typedef uint16_t Entry;
    static constexpr int kEntryBytes = 2, kUnitEntries = 8;
    static constexpr int kMaxCount = 15;
    static constexpr int kMaxK = 1023;          // topics 0 .. K, K being the padding entries'
    static constexpr int kWavesPerSimd = 5;
    static constexpr bool kOneEntryPerTopic = false;
    static __host__ __device__ __forceinline__ Entry make(int count, int topic) {
        return (Entry)(((uint32_t)count << 12) | ((uint32_t)topic << 2));
    }
    static __host__ __device__ __forceinline__ int entry_topic(Entry e) { return (int)((e >> 2) & 0x3ffu); }
    static __host__ __device__ __forceinline__ int entry_count(Entry e) { return (int)(e >> 12); }
    static __device__ __forceinline__ uint32_t word(const uint4& u, int j) {
        return (j >> 1) == 0 ? u.x : (j >> 1) == 1 ? u.y : (j >> 1) == 2 ? u.z : u.w;
    }
    static __device__ __forceinline__ int key(const uint4& u, int j) {
        const uint32_t d = word(u, j);
        return (j & 1) ? (int)__builtin_amdgcn_ubfe(d, 16, 12) : (int)(d & 0xffcu);
    }
    static __device__ __forceinline__ int count(const uint4& u, int j) {
        const uint32_t d = word(u, j);
        return (j & 1) ? (int)(d >> 28) : (int)__builtin_amdgcn_ubfe(d, 12, 4);
    }
};

// Unit `unit` of the row in slot `off`.  Every lane loads: a lane without entries reads the
// padding entries that the library keeps in the first 64 bytes of the slot buffer (no slot
// starts there).
__device__ __forceinline__ uint4 load_unit(const unsigned char* slots, uint32_t off, int unit, bool on) {
    static_assert(kRowHeader == 16, "a row's entries start one 16-byte unit into its slot");
    uint32_t at = on ? off + 1u + (uint32_t)unit : 0u;
    // the choice is made on the 32-bit unit number, before it becomes a 64-bit address
    asm volatile("" : "+v"(at));
    return *reinterpret_cast<const uint4*>(slots + (size_t)at * 16u);
}

// The same for a slot buffer smaller than 4 GiB.  `row_bytes` is the byte offset of the lane's
// first unit, `c` (a constant) the unit's number among the lane's units; a lane without that
// unit reads padding unit c (the buffer starts with kKeptUnits + 1 of them).
__device__ __forceinline__ uint4 load_unit_near(const unsigned char* slots, uint32_t row_bytes, int c, bool on) {
    uint32_t at = on ? row_bytes : 0u;
    asm volatile("" : "+v"(at));
    return *reinterpret_cast<const uint4*>(slots + (size_t)at + (size_t)(c * 16));
}

// A load and a store at a 32-bit byte offset from a base that is the same for the whole wave:
// the base stays in scalar registers and the offset is all a lane computes.
template <class T>
__device__ __forceinline__ T load_at(const void* base, uint32_t byte_offset) {
    return *reinterpret_cast<const T*>(reinterpret_cast<const unsigned char*>(base) + byte_offset);
}
template <class T>
__device__ __forceinline__ void store_at(void* base, uint32_t byte_offset, T v) {
    *reinterpret_cast<T*>(reinterpret_cast<unsigned char*>(base) + byte_offset) = v;
}

// Key of the entry that lies just before a unit in memory (a row's header ends in a padding
// entry, so this is always an entry).
template <class Layout>
__device__ __forceinline__ int key_before_unit(const unsigned char* unit_ptr) {
    typedef typename Layout::Entry Entry;
    return 4 * Layout::entry_topic(*reinterpret_cast<const Entry*>(unit_ptr - sizeof(Entry)));
}

// p*(k) is staged at the very start of the workgroup's LDS, so a topic's key (4 k) is the
// LDS address of its weight.
__device__ __forceinline__ float lds_float_at(uint32_t byte_address) {
    typedef __attribute__((address_space(3))) const float* lds_float_ptr;
    return *(lds_float_ptr)(uintptr_t)byte_address;
}

// Where the walk over a row finds p*(k) by the entry's key 4 k: in LDS ...
struct LdsWeights {
    __device__ __forceinline__ float operator()(uint32_t key) const { return lds_float_at(key); }
};
// ... or, when K is too large for that, in the workgroup's own strip of device memory (written by
// the workgroup itself before a barrier, and read through the CU's own cache).
struct FarWeights {
    const unsigned char* base;
    __device__ __forceinline__ float operator()(uint32_t key) const {
        return *reinterpret_cast<const float*>(base + key);
    }
};

// p1 = theta' p*' over the entries of one unit (Eq. 6), accumulated onto `acc` in entry order
// (each product is exact in fp64).  The token's own topic o weighs w_o in all its entries and
// its first entry counts one less: the token itself.  `prev_own`: the lanes whose entry before
// this unit belongs to their o; on return: those whose last entry of the unit does.  ("Own and
// first" is worked out on these lane masks, by the scalar unit.)
// This form leaves the sum at the unit's end only: every entry is added with its whole count,
// and the lanes whose first own entry lies in the unit give w_o back once, at the end.
template <class Layout, class Weights>
__device__ __forceinline__ void unit_sum(const Weights& weight_at, const uint4& raw, int o_key, float w_o,
                                         uint64_t& prev_own, double& acc) {
    constexpr int n = Layout::kUnitEntries;
    uint64_t first_here = 0;
#pragma unroll
    for (int h = 0; h < n; h += 4) {       // four gathers of p* on their way at a time
        int key[4];
        float w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            key[j] = Layout::key(raw, h + j);
            w[j] = weight_at((uint32_t)key[j]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool own = key[j] == o_key;
            const uint64_t own_lanes = __ballot(own);
            first_here |= own_lanes & ~prev_own;
            prev_own = own_lanes;
            acc = fma((double)Layout::count(raw, h + j), (double)(own ? w_o : w[j]), acc);
        }
    }
    acc -= __builtin_amdgcn_inverse_ballot_w64(first_here) ? (double)w_o : 0.0;
}

// The same with the running sum after every entry and the entries' keys kept (the first own
// entry counts one less where it stands).
template <class Layout, class Weights>
__device__ __forceinline__ void unit_prefix_sums(const Weights& weight_at, const uint4& raw, int o_key, float w_o,
                                                 uint64_t& prev_own, double& acc, double* sums, int* keys) {
    constexpr int n = Layout::kUnitEntries;
#pragma unroll
    for (int j = 0; j < n; ++j) {
        const int key = Layout::key(raw, j);
        const bool own = key == o_key;
        const uint64_t own_lanes = __ballot(own);
        const bool first = __builtin_amdgcn_inverse_ballot_w64(own_lanes & ~prev_own);
        prev_own = own_lanes;
        acc = fma((double)(Layout::count(raw, j) - (first ? 1 : 0)),
                  (double)(own ? w_o : weight_at((uint32_t)key)), acc);
        sums[j] = acc;
        keys[j] = key;
    }
}

// What the lanes of a group need of their token for the walk, read back from its record.
struct RowCtx {
    uint32_t off;           // slot of the row
    int o_key;              // 4 * current topic (a topic's key is its byte offset in p*)
    float w_o;
};

__device__ __forceinline__ RowCtx row_ctx(const TokenRec* rec) {
    const int4 head = *reinterpret_cast<const int4*>(rec);
    RowCtx r;
    r.off = (uint32_t)head.x; r.o_key = head.z << 2; r.w_o = __int_as_float(head.w);
    return r;
}

// Row total S (Eq. 7), the draw x = u (S + Q'), and whether this lane's entries hold it.
struct RowDraw {
    double S, x, y;         // y = x - (sum of the group's sub-lanes before this one)
    bool sparse, hit;
};

template <int kLanes>
__device__ __forceinline__ RowDraw row_draw(double lane_sum, const TokenRec* rec, int sl, int lane) {
    RowDraw d;
    const double incl = group_inclusive_sum<kLanes>(lane_sum);
    const double excl = group_previous<kLanes>(incl, sl);
    // (the lane that holds the group's total is worked out here, every time: hoisted out of
    // the loop over passes, one such constant per shape would each hold a register for good)
    asm volatile("" : "+v"(lane));
    d.S = __shfl(incl, group_last_lane<kLanes>(lane), kWave);
    const double2 uq = *reinterpret_cast<const double2*>(&rec->u);     // the uniform, and Q'
    d.x = uq.x * (d.S + uq.y);
    d.sparse = d.x < d.S;
    d.hit = d.sparse && (incl > d.x) && !(excl > d.x);
    d.y = d.x - excl;
    return d;
}

// A token whose draw falls into the dense bucket p2: recorded once, by its first sub-lane.
__device__ __forceinline__ void record_dense(TokenRec* rec, int sl, const RowDraw& d) {
    if (!d.sparse && sl == 0) {
        rec->nnz = kDrawDense;
        rec->u = d.x - d.S;
    }
}

// Rows whose sub-lanes own at most kUnits units, already loaded (sub-lane sl owns the units from
// sl * kUnits on).  Every lane keeps its sum at the end of each unit; the lane that holds
// the draw records which unit holds it and the rest of the draw there.
// Rows with one entry per topic, already loaded: every lane keeps the running sum after each of
// its entries, and the lane that holds the draw finds its entry at once.
template <class Layout, int kLanes, int kUnits, class Weights>
__device__ __forceinline__ void row_pass_searched(const Weights& weight_at, TokenRec* rec, int sl,
                                                  const uint4* raw, int lane) {
    constexpr int UE = Layout::kUnitEntries, n = kUnits * UE;
    const RowCtx r = row_ctx(rec);
    double sums[n];
    double acc = 0.0;
#pragma unroll
    for (int c = 0; c < kUnits; ++c) {
        int key[UE];
        float w[UE];
#pragma unroll
        for (int j = 0; j < UE; ++j) {
            key[j] = Layout::key(raw[c], j);
            w[j] = weight_at((uint32_t)key[j]);
        }
#pragma unroll
        for (int j = 0; j < UE; ++j) {
            const bool own = key[j] == r.o_key;
            acc = fma((double)(Layout::count(raw[c], j) - (own ? 1 : 0)), (double)(own ? r.w_o : w[j]), acc);
            sums[c * UE + j] = acc;
        }
    }
    const RowDraw d = row_draw<kLanes>(acc, rec, sl, lane);
    // smallest entry whose sum exceeds y (the sums never decrease)
    uint32_t entry = Layout::word(raw[kUnits - 1], UE - 1);
#pragma unroll
    for (int i = n - 2; i >= 0; --i)
        if (sums[i] > d.y) entry = Layout::word(raw[i / UE], i % UE);
    if (__builtin_expect(__ballot(d.hit && !(acc > d.y)) != 0, 0)) {   // rounding left no sum above the draw:
        asm volatile("");                            // (a branch of its own: it is almost never taken)
        if (d.hit && !(acc > d.y)) {                 // take the lane's last entry with weight
            double before = 0.0;
#pragma unroll
            for (int i = 0; i < n; ++i) {
                if (sums[i] > before) entry = Layout::word(raw[i / UE], i % UE);
                before = sums[i];
            }
        }
    }
    if (d.hit) {
        rec->off = (uint32_t)Layout::entry_topic(entry);
        rec->nnz = kDrawTopic;
    }
    record_dense(rec, sl, d);
}

template <class Layout, int kLanes, int kUnits, class Weights>
__device__ __forceinline__ void row_pass_kept(const Weights& weight_at, TokenRec* rec, int sl,
                                              const uint4* raw, int lane) {
    const int first_unit = sl * kUnits;
    if constexpr (Layout::kOneEntryPerTopic) {
        row_pass_searched<Layout, kLanes, kUnits>(weight_at, rec, sl, raw, lane);
        return;
    }
    const RowCtx r = row_ctx(rec);
    // does the entry before this lane's first one belong to the token's own topic?  (the
    // previous sub-lane's last entry; a sub-lane past the row's end holds padding entries)
    const int before = group_previous_int<kLanes>(Layout::key(raw[kUnits - 1], Layout::kUnitEntries - 1));
    uint64_t prev_own = __ballot(sl > 0 && before == r.o_key);
    double at_end[kUnits];
    double acc = 0.0;
#pragma unroll
    for (int c = 0; c < kUnits; ++c) {
        unit_sum<Layout>(weight_at, raw[c], r.o_key, r.w_o, prev_own, acc);
        at_end[c] = acc;
    }
    const RowDraw d = row_draw<kLanes>(acc, rec, sl, lane);
    // first unit whose end exceeds y (the sums never decrease), and the sum before it
    int unit = kUnits - 1;
#pragma unroll
    for (int c = kUnits - 2; c >= 0; --c)
        if (at_end[c] > d.y) unit = c;
    if (__builtin_expect(__ballot(d.hit && !(acc > d.y)) != 0, 0)) {   // rounding left no sum above the draw:
        asm volatile("");                            // (a branch of its own: it is almost never taken)
        if (d.hit && !(acc > d.y)) {                 // take the lane's last unit with weight
            double before_unit = 0.0;
#pragma unroll
            for (int c = 0; c < kUnits; ++c) {
                if (at_end[c] > before_unit) unit = c;
                before_unit = at_end[c];
            }
        }
    }
    double base = 0.0;
#pragma unroll
    for (int c = 1; c < kUnits; ++c)
        if (unit >= c) base = at_end[c - 1];
    if (d.hit) {
        rec->off = r.off + 1u + (uint32_t)(first_unit + unit);
        rec->nnz = kDrawInUnit;
        rec->u = d.y - base;
    }
    record_dense(rec, sl, d);
}

// The entry of one unit that holds the draw y (measured from the unit's start): the first
// whose running sum exceeds y, else (rounding) the last one with weight.  One token per lane.
template <class Layout, bool kNear, class Weights>
__device__ __forceinline__ int topic_in_unit(const Weights& weight_at, const unsigned char* slots, uint32_t unit,
                                             int o_key, float w_o, double y) {
    constexpr int n = Layout::kUnitEntries;
    const unsigned char* p = kNear ? slots + (size_t)(uint32_t)(unit << 4) : slots + (size_t)unit * 16u;
    const uint4 raw = *reinterpret_cast<const uint4*>(p);
    uint64_t prev_own = __ballot(key_before_unit<Layout>(p) == o_key);
    double acc = 0.0;
    int found = -1, last = Layout::key(raw, 0);     // keys: the first above y, the last with weight
#pragma unroll
    for (int j = 0; j < n; ++j) {
        const int key = Layout::key(raw, j);
        const uint64_t own_lanes = __ballot(key == o_key);
        const bool own = __builtin_amdgcn_inverse_ballot_w64(own_lanes);
        const bool first = __builtin_amdgcn_inverse_ballot_w64(own_lanes & ~prev_own);
        prev_own = own_lanes;
        const double before = acc;
        acc = fma((double)(Layout::count(raw, j) - (first ? 1 : 0)),
                  (double)(own ? w_o : weight_at((uint32_t)key)), acc);
        if (acc > before) last = key;
        if (found < 0 && acc > y) found = key;
    }
    return (found >= 0 ? found : last) >> 2;
}

// Rows too long for the kept shapes, one per wave (sub-lane = lane): one walk for the sums, a
// second one over the hit lane's entries.  Lane l owns the units [n l, n (l + 1)).
template <class Layout, class Weights>
__device__ __forceinline__ void row_pass_long(const Weights& weight_at, const unsigned char* slots, TokenRec* rec,
                                              int lane) {
    constexpr int UE = Layout::kUnitEntries;
    const RowCtx r = row_ctx(rec);
    const int n_units = rec->nnz, n = (n_units + kWave - 1) / kWave;
    const int u0 = lane * n;
    // the entry before the lane's first one (lanes past the row's end have no entries at all)
    const bool own_before = u0 < n_units &&
        key_before_unit<Layout>(slots + ((size_t)r.off + 1u + (size_t)u0) * 16u) == r.o_key;
    uint64_t prev_own = __ballot(own_before);
    double acc = 0.0;
    for (int c = 0; c < n; ++c)
        unit_sum<Layout>(weight_at, load_unit(slots, r.off, u0 + c, u0 + c < n_units), r.o_key, r.w_o, prev_own,
                         acc);
    const RowDraw d = row_draw<kWave>(acc, rec, lane, lane);
    if (__ballot(d.hit) != 0) {
        bool found = false;
        int k_sel = 0, last_k = 0;
        prev_own = __ballot(own_before);
        acc = 0.0;
        for (int c = 0; c < n; ++c) {
            double sums[UE];
            int keys[UE];
            const double before_unit = acc;
            unit_prefix_sums<Layout>(weight_at, load_unit(slots, r.off, u0 + c, d.hit && u0 + c < n_units),
                                     r.o_key, r.w_o, prev_own, acc, sums, keys);
#pragma unroll
            for (int j = 0; j < UE; ++j) {
                const double before = (j == 0) ? before_unit : sums[j - 1];
                if (!found && sums[j] > d.y) { k_sel = keys[j] >> 2; found = true; }
                if (sums[j] > before) last_k = keys[j] >> 2;
            }
        }
        if (d.hit) {
            rec->off = (uint32_t)(found ? k_sel : last_k);
            rec->nnz = kDrawTopic;
        }
    }
    record_dense(rec, lane, d);
}

// kFar: K is too large for p* to fit a workgroup's LDS.  p* of the workgroup's tile then lives in
// the workgroup's own strip of device memory (the prefix sums and the records stay in LDS), and
// the launch has as many workgroups as there are strips, each taking every grid-th tile.
// kNear: every byte of the slot buffer has a 32-bit offset; a pass then finds its units with
// 32-bit arithmetic (one offset per lane, the unit's place in the load's own offset field).
template <int kWaves, class Layout, bool kFar = false, bool kNear = false>
// Six waves per SIMD (80 VGPRs): the walk hides HBM latency by occupancy as well as by the
// early loads.
__attribute__((amdgpu_waves_per_eu(Layout::kWavesPerSimd)))
__global__ __launch_bounds__(kWaves * kWave) void sample_kernel(const SampleArgs a) {
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int kGroup = dense_group(kWaves);
    const int K = a.K, Kpad = a.Kpad, ng = Kpad / kGroup;
    const size_t pstar_lds = kFar ? 0 : (size_t)Kpad * 4;
    float* pstar = kFar ? a.far_pstar + (size_t)blockIdx.x * (size_t)Kpad : reinterpret_cast<float*>(lds);
    double* cp = reinterpret_cast<double*>(lds + pstar_lds);
    const int tid = (int)threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);      // wave-uniform, in an SGPR
    unsigned char* wave_base = lds + pstar_lds + (size_t)((ng + 1) & ~1) * 8;
    TokenRec* my_rec = reinterpret_cast<TokenRec*>(wave_base) + wave * kWave;
    typedef typename std::conditional<kFar, FarWeights, LdsWeights>::type Weights;
    Weights weight_at;
    if constexpr (kFar) weight_at.base = reinterpret_cast<const unsigned char*>(pstar);

    // The workgroup's tiles: one, or (large K only) a run of small ones.  What says where the
    // run starts and ends is worked out again where it is needed rather than kept through the
    // token phase, whose registers are all taken.
    // Runs are dealt evenly among the other workgroups in launch order (the runs wait for memory
    // most of the time, the large tiles keep the arithmetic units busy: side by side on a CU they
    // fill each other's gaps): of the workgroups before b, floor(b * n_runs / grid) take a run.
    constexpr bool kRuns = kWaves == 12 && !kFar;
    auto runs_before = [&](int b) {
        const int n_runs = (int)gridDim.x - a.n_single;
        return (int)((int64_t)b * n_runs / (int64_t)gridDim.x);
    };
    auto in_run = [&]() { return kRuns && runs_before((int)blockIdx.x + 1) > runs_before((int)blockIdx.x); };
    auto first_tile = [&]() {
        const int before = kRuns ? runs_before((int)blockIdx.x) : 0;
        return in_run() ? a.n_single + before * a.run_tiles : (int)blockIdx.x - before;
    };
    auto last_tile = [&]() { return in_run() ? min(first_tile() + a.run_tiles, a.n_tiles) : first_tile() + 1; };
    double* group_sum = reinterpret_cast<double*>(wave_base + (size_t)kWaves * kWave * sizeof(TokenRec));
    uint32_t* changed = reinterpret_cast<uint32_t*>(group_sum + ((ng + 1) & ~1));
    if (in_run()) {
        for (int w = tid; w < (ng + 31) / 32; w += kWaves * kWave) changed[w] = 0u;
    }
    for (int ti = kFar ? (int)blockIdx.x : first_tile();;) {
    Tile tl = a.tiles[ti];                 // the same for every lane: keep it in SGPRs
    tl.word = __builtin_amdgcn_readfirstlane(tl.word);
    tl.begin = __builtin_amdgcn_readfirstlane(tl.begin);
    tl.count = __builtin_amdgcn_readfirstlane(tl.count);
    // the word's row of phi: 16-bit or 32-bit cells, the same for the whole workgroup
    const int wide_row = __builtin_amdgcn_readfirstlane(tl.whole);    // (kept in the tile: one load less in the chain)
    const bool wide = wide_row >= 0;
    const unsigned char* phi_cells = wide ? reinterpret_cast<const unsigned char*>(a.phi.wide)
                                          : reinterpret_cast<const unsigned char*>(a.phi.narrow);
    const size_t phi_cell0 = (size_t)(wide ? wide_row : tl.word) * (size_t)K;
    const uint32_t phi_shift = wide ? 2u : 1u, phi_mask = wide ? 0xffffffffu : 0xffffu;

    if (kRuns && ti > first_tile()) {
        const Tile prev = a.tiles[ti - 1];
        const int prev_begin = __builtin_amdgcn_readfirstlane(prev.begin);
        const int prev_count = __builtin_amdgcn_readfirstlane(prev.count);
        // ---- p* of the run's previous word becomes p* of this one.  Both words have all their
        // tokens in their tile, so a cell of phi is non-zero exactly for the topics of the
        // tile's tokens: only those cells differ from beta / (n_k + beta V).  Every changed cell
        // gets the value a fresh staging would give it, and the sums of the groups that hold
        // one are added up again in the same order, so the result is the fresh staging's, bit
        // for bit.
        for (int idx = tid; idx < prev_count; idx += kWaves * kWave) {
            const int k = (int)a.z_cur[prev_begin + idx];
            pstar[k] = (float)((0.0 + a.beta) / ((double)a.n_k[k] + a.beta_V));
            atomicOr(&changed[(k / kGroup) >> 5], 1u << ((k / kGroup) & 31));
        }
        __syncthreads();
        const uint16_t* phi_v = reinterpret_cast<const uint16_t*>(phi_cells) + phi_cell0;   // (never a wide row)
        for (int idx = tid; idx < tl.count; idx += kWaves * kWave) {
            const int k = (int)a.z_cur[tl.begin + idx];
            pstar[k] = (float)(((double)phi_v[k] + a.beta) / ((double)a.n_k[k] + a.beta_V));
            atomicOr(&changed[(k / kGroup) >> 5], 1u << ((k / kGroup) & 31));
        }
        __syncthreads();
        for (int g = tid; g < ng; g += kWaves * kWave)
            if ((changed[g >> 5] >> (g & 31)) & 1u) {
                double s = 0.0;
#pragma unroll
                for (int j = 0; j < kGroup; ++j) s += (double)pstar[g * kGroup + j];
                group_sum[g] = s;
            }
        __syncthreads();
        if (wave == 0) {
            for (int w = lane; w < (ng + 31) / 32; w += kWave) changed[w] = 0u;
            double carry = 0.0;
            for (int base = 0; base < ng; base += kWave) {
                const int g = base + lane;
                double x = (g < ng) ? group_sum[g] : 0.0;
                x = wave_inclusive_sum(x) + carry;
                if (g < ng) cp[g] = x;
                carry = read_lane(x, kWave - 1);
            }
        }
        __syncthreads();
    } else {
    // ---- stage p*(k) = (phi_kv + beta)/(n_k + beta V) as fp32 (Eq. 8)
    if (wide) {
        const int32_t* phi_v = reinterpret_cast<const int32_t*>(phi_cells) + phi_cell0;
        for (int k = tid; k < Kpad; k += kWaves * kWave) {
            float w = 0.f;
            if (k < K) w = (float)(((double)phi_v[k] + a.beta) / ((double)a.n_k[k] + a.beta_V));
            pstar[k] = w;
        }
    } else {
        const uint16_t* phi_v = reinterpret_cast<const uint16_t*>(phi_cells) + phi_cell0;
        for (int k = tid; k < Kpad; k += kWaves * kWave) {
            float w = 0.f;
            if (k < K) w = (float)(((double)phi_v[k] + a.beta) / ((double)a.n_k[k] + a.beta_V));
            pstar[k] = w;
        }
    }
    __syncthreads();
    for (int g = tid; g < ng; g += kWaves * kWave) {
        double s = 0.0;
#pragma unroll
        for (int j = 0; j < kGroup; ++j) s += (double)pstar[g * kGroup + j];
        cp[g] = s;
        if (in_run()) group_sum[g] = s;
    }
    __syncthreads();
    if (wave == 0) {                       // inclusive prefix over the group sums
        double carry = 0.0;
        for (int base = 0; base < ng; base += kWave) {
            const int g = base + lane;
            double x = (g < ng) ? cp[g] : 0.0;
            x = wave_inclusive_sum(x) + carry;
            if (g < ng) cp[g] = x;
            carry = read_lane(x, kWave - 1);
        }
    }
    __syncthreads();
    }

    // a pass shape's lane geometry: token of the lane relative to the pass's first, the lane's
    // place inside its group, its first unit of entries
    int geo_shape = -1, geo_rel = 0, geo_sl = 0, geo_q0 = 0;
    // A wave takes up to 64 tokens at a time.  A tile too small to give every wave such a batch
    // is dealt out in smaller batches, so that all waves work on it side by side: the passes
    // of one batch follow each other, each waiting for its rows.
    const int batch = kWaves == 4 ? kWave
                    : min(kWave, max(kMinBatch, ((tl.count + kWaves - 1) / kWaves + 3) & ~3));
    const int n_batches = (tl.count + batch - 1) / batch;
    for (int b = wave; b < n_batches; b += kWaves) {
        // ---- one token per lane: token, uniform, own-count correction
        const int idx = b * batch + lane;
        const bool valid = lane < batch && idx < tl.count;
        TokenRec mine;
        mine.off = 0; mine.nnz = 0; mine.o = 0; mine.w_o = 0.f; mine.u = 0.0; mine.Qp = 0.0;
        double delta = 0.0;
        // What the per-token phases read of the kernel's arguments is fetched from the argument
        // block again in every batch (scalar loads) instead of being kept in scalar registers
        // through the passes: there are not enough of those, and what does not fit is parked in
        // lanes of a vector register, every read of which takes a vector issue slot.
        // (SampleArgs is the kernel's only parameter, so the argument block starts with it.)
        typedef __attribute__((address_space(4))) const SampleArgs* ArgsPtr;
        ArgsPtr ka = (ArgsPtr)__builtin_amdgcn_kernarg_segment_ptr();
        asm volatile("" : "+s"(ka));
        if (valid) {
            // (the tile's part of every per-token array starts at a scalar base)
            mine.off = load_at<uint32_t>(ka->tok_slot + tl.begin, (uint32_t)idx << 2);
            mine.o = (int)load_at<uint16_t>(ka->z_cur + tl.begin, (uint32_t)idx << 1);
            const uint64_t id = (uint64_t)load_at<uint32_t>(ka->tok_id + tl.begin, (uint32_t)idx << 2);
            // the row's length sits in front of its entries: this read also brings the row's
            // first line on its way
            const uint32_t entries = kNear ? load_at<uint32_t>(a.slots, mine.off << 4)
                                           : *reinterpret_cast<const uint32_t*>(a.slots + (size_t)mine.off * 16u);
            mine.nnz = (int)((entries + (uint32_t)(Layout::kUnitEntries - 1)) / (uint32_t)Layout::kUnitEntries);
            // (the seed too: the ten rounds' keys are then made where they are used, by the scalar
            // unit, and not once per kernel)
            mine.u = token_uniform(ka->seed, ka->iter, id);
            // the token itself is taken out of phi and n_k at its own topic
            // (its cell of phi, of either width, is cut out of the aligned dword that holds it)
            const size_t row_byte = phi_cell0 << phi_shift;        // the word's row: scalar
            const uint32_t own_byte = ((uint32_t)row_byte & 3u) + ((uint32_t)mine.o << phi_shift);
            const uint32_t own_dword = load_at<uint32_t>(phi_cells + (row_byte & ~(size_t)3), own_byte & ~3u);
            const int32_t phi_own = (int32_t)((own_dword >> ((own_byte & 2u) << 3)) & phi_mask);
            mine.w_o = (float)(((double)(phi_own - 1) + ka->beta) /
                               ((double)(ka->n_k[mine.o] - 1) + ka->beta_V));
            delta = (double)mine.w_o - (double)pstar[mine.o];
            // cp[ng - 1] = sum_k p*(k), read from LDS where it is needed; Q = alpha sum (Eq. 7)
            mine.Qp = ka->alpha * (cp[ng - 1] + delta);
        }
        my_rec[lane] = mine;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- one token per group of 4 .. 64 lanes.  A pass takes the next 16, 8, 4, 2 or 1
        // tokens, as many as lets every lane own at most kKeptUnits units; the rows of the
        // following pass are requested from memory before this one is worked on.
        // Shapes of a pass (lanes per token, units per lane); a row may have up to
        // lanes * units * (entries per unit) entries:
        //   0 (4,1)   1 (4,2)   2 (4,3)   3 (8,2)   4 (8,3)   5 (16,2)   6 (16,3)
        //   7 (32,2)   8 (32,3)   9 (64,2)   10 (64,3)   11 = one longer row, walked twice by the wave
        // Which tokens of the batch have rows beyond each of these lengths (lanes past the
        // batch's end hold nnz = 0): the shape of every pass follows from these masks.
        const int n_here = min(batch, tl.count - b * batch);
        static_assert(kKeptUnits == 3, "the pass shapes assume three kept units per lane");
        const uint64_t over_4_1 = __ballot(mine.nnz > 4), over_4_2 = __ballot(mine.nnz > 8);
        const uint64_t over_4_3 = __ballot(mine.nnz > 12), over_8_2 = __ballot(mine.nnz > 16);
        const uint64_t over_8_3 = __ballot(mine.nnz > 24), over_16_2 = __ballot(mine.nnz > 32);
        const uint64_t over_16_3 = __ballot(mine.nnz > 48), over_32_2 = __ballot(mine.nnz > 64);
        const uint64_t over_32_3 = __ballot(mine.nnz > 96), over_64_2 = __ballot(mine.nnz > 128);
        const uint64_t over_64_3 = __ballot(mine.nnz > 192);
        auto any = [](uint64_t mask, int t0, uint32_t window) {      // 1 if a token of the window is set
            const uint32_t w = (uint32_t)(mask >> t0) & window;
            return min(1, (int)__builtin_popcount(w));      // stays scalar arithmetic
        };
        auto shape_at = [&](int t0) {
            if (!any(over_4_3, t0, 0xffffu)) return any(over_4_1, t0, 0xffffu) + any(over_4_2, t0, 0xffffu);
            if (!any(over_8_3, t0, 0xffu)) return 3 + any(over_8_2, t0, 0xffu);
            if (!any(over_16_3, t0, 0xfu)) return 5 + any(over_16_2, t0, 0xfu);
            if (!any(over_32_3, t0, 0x3u)) return 7 + any(over_32_2, t0, 0x3u);
            if (!any(over_64_3, t0, 0x1u)) return 9 + any(over_64_2, t0, 0x1u);
            return 11;
        };
        auto lanes_log2 = [](int shape) { return (int)((0x666554433222ull >> (4 * shape)) & 0xfull); };
        auto units_of = [](int shape) { return (int)((0x032323232321ull >> (4 * shape)) & 0xfull); };
        // where a pass's rows are, and the loads of the units its lanes keep.  `rec` is the
        // record of the lane's token, `sl` the lane's place inside its group.  A pass that
        // would run past the batch's 64 records works on the last one several times over.
        auto request = [&](int t0, int shape, TokenRec*& rec, int& sl, uint4* raw, bool live) {
            const int nu = units_of(shape);
            if (shape != geo_shape) {       // the lanes' places change only with the shape
                const int lg = lanes_log2(shape);
                const int g = lg < 4 ? 4 - lg : 0, hs = lg < 4 ? 4 : lg;    // interleave, run length
                geo_shape = shape;
                geo_rel = ((lane >> hs) << g) | (lane & ((1 << g) - 1));
                geo_sl = (lane & ((1 << hs) - 1)) >> g;
                geo_q0 = geo_sl * nu;        // the lane's first unit
            }
            sl = geo_sl;
            rec = my_rec + min(t0 + geo_rel, kWave - 1);
            const uint2 where = *reinterpret_cast<const uint2*>(rec);
            // units the lane loads: those of the shape that the row still has from its first on
            const int n_mine = live ? min((int)where.y - geo_q0, nu) : 0;
            if constexpr (kNear) {
                const uint32_t row_bytes = (where.x + 1u + (uint32_t)geo_q0) << 4;
#pragma unroll
                for (int c = 0; c < kKeptUnits; ++c)
                    raw[c] = load_unit_near(a.slots, row_bytes, c, c < n_mine);
            } else {
#pragma unroll
                for (int c = 0; c < kKeptUnits; ++c)
                    raw[c] = load_unit(a.slots, where.x, geo_q0 + c, c < n_mine);
            }
        };
        int t_next = 0, shape_next = shape_at(0), sl_next;
        TokenRec* rec_next;
        // one pass: `mine_raw` holds its rows, already requested; the following pass's rows
        // go to `next_raw`.  The two buffers swap roles from pass to pass.
        auto pass = [&](uint4* mine_raw, uint4* next_raw) {
            const int shape = shape_next, sl = sl_next;
            TokenRec* rec = rec_next;
            t_next += kWave >> lanes_log2(shape);
            // The request is made whether or not a pass follows (after the batch's last pass
            // every lane loads padding units): the number of loads in flight behind this
            // pass's own is then the same on every path, and the pass waits for its own rows
            // only, not for the first of the following pass's as well.
            const int t_req = min(t_next, kWave - 1);
            shape_next = shape_at(t_req);
            request(t_req, shape_next, rec_next, sl_next, next_raw, t_next < n_here);
            switch (shape) {
            case 0: row_pass_kept<Layout, 4, 1>(weight_at, rec, sl, mine_raw, lane); break;
            case 1: row_pass_kept<Layout, 4, 2>(weight_at, rec, sl, mine_raw, lane); break;
            case 2: row_pass_kept<Layout, 4, 3>(weight_at, rec, sl, mine_raw, lane); break;
            case 3: row_pass_kept<Layout, 8, 2>(weight_at, rec, sl, mine_raw, lane); break;
            case 4: row_pass_kept<Layout, 8, 3>(weight_at, rec, sl, mine_raw, lane); break;
            case 5: row_pass_kept<Layout, 16, 2>(weight_at, rec, sl, mine_raw, lane); break;
            case 6: row_pass_kept<Layout, 16, 3>(weight_at, rec, sl, mine_raw, lane); break;
            case 7: row_pass_kept<Layout, 32, 2>(weight_at, rec, sl, mine_raw, lane); break;
            case 8: row_pass_kept<Layout, 32, 3>(weight_at, rec, sl, mine_raw, lane); break;
            case 9: row_pass_kept<Layout, 64, 2>(weight_at, rec, sl, mine_raw, lane); break;
            case 10: row_pass_kept<Layout, 64, 3>(weight_at, rec, sl, mine_raw, lane); break;
            default: row_pass_long<Layout>(weight_at, a.slots, rec, lane); break;
            }
        };
        uint4 raw_a[kKeptUnits], raw_b[kKeptUnits];
        request(0, shape_next, rec_next, sl_next, raw_a, true);
        while (t_next < n_here) {
            pass(raw_a, raw_b);
            if (t_next < n_here) pass(raw_b, raw_a);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- one token per lane again: the entry inside the unit that holds the draw, or the
        // dense bucket; store
        // (the token's topic and corrected weight are read back from its record rather than
        // kept in registers across the passes)
        if (lane < batch && b * batch + lane < tl.count) {
            const TokenRec* rec = &my_rec[lane];
            const int4 head = *reinterpret_cast<const int4*>(rec);     // off, kind, o, w_o
            const float w_o = __int_as_float(head.w);
            int z_new = head.x;
            if (head.y == kDrawInUnit)
                z_new = topic_in_unit<Layout, kNear>(weight_at, a.slots, (uint32_t)head.x, head.z << 2, w_o, rec->u);
            if (head.y == kDrawDense)
                z_new = dense_bucket_search<kGroup>(pstar, cp, K, ng, ka->alpha, rec->u, head.z, w_o,
                                                    (double)w_o - (double)pstar[head.z]);
            store_at<uint16_t>(ka->z_next + tl.begin, (uint32_t)(b * batch + lane) << 1, (uint16_t)z_new);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    ti += kFar ? (int)gridDim.x : 1;
    if (kFar ? ti >= a.n_tiles : (!kRuns || ti >= last_tile())) break;
    __syncthreads();                // every wave is done with this word's p*
    }
}

// Initial topics: z = floor(u(seed, 0, token) K), in word-major order.
__global__ void init_topics_kernel(const int32_t* tok_id, uint16_t* z, int64_t T, int32_t K,
                                   uint64_t seed) {
    const int64_t pos = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pos >= T) return;
    const double u = token_uniform(seed, 0u, (uint64_t)(uint32_t)tok_id[pos]);
    int k = (int)(u * (double)K);
    if (k > K - 1) k = K - 1;
    z[pos] = (uint16_t)k;
}

__global__ void philox_uniform_kernel(uint64_t seed, uint32_t iter, uint64_t token0, int64_t n,
                                      double* out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = token_uniform(seed, iter, token0 + (uint64_t)i);
}

}  // namespace mlda
