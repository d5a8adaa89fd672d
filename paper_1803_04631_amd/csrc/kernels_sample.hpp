// Sampling kernel: one pass of the sparsity-aware sampler (paper Section 6.1, Eq. 6-8,
// Algorithm 2) over word-sorted tokens.
//
// Mapping to gfx950 (the paper's own mapping, one 32-wide warp per sampler with 32-way
// index trees, was made for NVIDIA warps; measured here, a whole 64-lane wave per token is
// bound by VALU issue, not by HBM):
//   - a workgroup owns one tile = up to 1024 (4096 for large K) consecutive tokens of ONE
//     word and stages that word's p*(k) (Eq. 8) once in LDS as fp32, with fp64 prefix sums
//     over groups of 4 (or 16) topics (Section 6.1.2: samplers of a block share the word's data);
//   - each wave takes 64 tokens at a time (fewer when a large-K tile is too small to give every
//     wave that many).  What is per token and needs no cooperation is
//     done one token per LANE: the Philox uniform, the token's own-count correction of
//     p*(o), and the search in the dense bucket p2 (binary search over the group prefixes,
//     then the group's topics);
//   - the walk over the token's sparse theta row (S and the p1 prefix sums, Eq. 6-7) is done
//     by a GROUP of 4, 8, 16, 32 or 64 lanes per token, chosen per pass from the row lengths
//     so that a lane owns at most twelve entries (16, 8, 4, 2 or 1 tokens per pass: the fixed
//     cost of a pass is shared by as many tokens as their rows allow).  Groups narrower than
//     a DPP row of 16 lanes are interleaved inside the row (4 or 2 tokens side by side), so
//     that plain row shifts scan every group at once.  Every lane owns a contiguous run of
//     entries, loaded four at a time, accumulates them in fp64 in registers, and a DPP scan
//     over the group gives the prefix over lanes.  The lane whose range holds the draw finds
//     "the smallest k whose prefix exceeds it" (Section 6.1.1) among its own entries.  Rows
//     of more than 768 entries are walked twice by a whole wave.  Token parameters and
//     results travel between the per-lane and per-group phases through small per-wave LDS
//     records;
//   - the row walk is a chain of dependent loads (record, then a random row in HBM), so the
//     loads of the next pass are issued before the current pass is worked on.
#pragma once
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
    // whose first word is the row's length, then holds the entries in one of the two layouts
    // below (SplitRows / PackedRows); padding entries hold count 0 and topic K
    const unsigned char* slots;
    PhiView phi;
    const int32_t* n_k;         // [K]
    int32_t K, Kpad;            // Kpad = K+1 rounded up to a multiple of the dense group: p*(K..Kpad-1) = 0
    double alpha, beta, beta_V;
    uint64_t seed;
    uint32_t iter;
};

constexpr int kRowHeader = 16;  // bytes before a theta row's entries
// Topics per fp64 prefix group of the dense bucket: 4 where LDS has room (workgroups of four
// waves, K <= 2048), 16 for the large-K workgroups of twelve waves.
__host__ __device__ constexpr int dense_group(int waves) { return waves == 4 ? 4 : 16; }
constexpr int kKeptQuads = 3;   // quads (of four entries) a lane keeps in registers at most
constexpr int kMinBatch = 8;    // tokens a wave takes at a time at least

// Once a token's pass has read its record, the record takes the result back to the per-lane
// phase: the new topic (or -1 for "dense bucket") in `off`, the dense draw position in `u`.
struct __align__(16) TokenRec { // per-lane phase -> per-group phase, 32 bytes
    uint32_t off;               // slot offset of the token's theta row, 16-byte units
    int32_t nnz;
    int32_t o;                  // current topic
    float w_o;                  // p*(o) with the token itself removed
    double u;
    double Qp;                  // alpha * sum_k p*'(k)
};

// LDS bytes of sample_kernel<kWaves> for a given Kpad.
__host__ __device__ constexpr size_t sample_lds_bytes(int Kpad, int waves) {
    return (size_t)Kpad * 4 + (size_t)((Kpad / dense_group(waves) + 1) & ~1) * 8 +
           (size_t)waves * kWave * sizeof(TokenRec);
}

// Dense bucket (p2 = alpha p*', Eq. 6): smallest k with alpha * prefix'(k) > y, where
// prefix' is the prefix sum of p* with the entry of the token's own topic o replaced by
// w_o (delta = w_o - p*(o)).  One lane per token.
template <int kGroup>
__device__ __forceinline__ int dense_bucket_search(const float* pstar, const double* cp, int K,
                                                   int ng, double alpha, double y, int o,
                                                   float w_o, double delta) {
    int lo = 0, hi = ng;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        const double pre = cp[mid] + ((mid * kGroup + (kGroup - 1) >= o) ? delta : 0.0);
        if (alpha * pre > y) hi = mid; else lo = mid + 1;
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

// Layout of a theta row inside its slot, 6 bytes per entry: int32 counts[round4(nnz)] then
// uint16 topics[round4(nnz)].  Always usable.
struct SplitRows {
    static constexpr int kEntryBytes = 6;
    static constexpr int kWavesPerSimd = 5;
    struct Raw {            // four consecutive entries as they come from memory
        int4 c;             // counts
        uint2 t;            // topics, two per dword
    };
    static __device__ __forceinline__ Raw load(const unsigned char* slots, uint32_t off, int nnz,
                                               int e, bool on, int K) {
        Raw q;
        q.c = make_int4(0, 0, 0, 0);
        q.t = make_uint2((uint32_t)K | ((uint32_t)K << 16), (uint32_t)K | ((uint32_t)K << 16));
        if (on) {
            const int32_t* cnt = reinterpret_cast<const int32_t*>(slots + (size_t)off * 16u + kRowHeader);
            const uint16_t* top = reinterpret_cast<const uint16_t*>(cnt + ((nnz + 3) & ~3));
            q.c = *reinterpret_cast<const int4*>(cnt + e);
            q.t = *reinterpret_cast<const uint2*>(top + e);
        }
        return q;
    }
    static __device__ __forceinline__ int count(const Raw& q, int j) {
        return j == 0 ? q.c.x : j == 1 ? q.c.y : j == 2 ? q.c.z : q.c.w;
    }
    static __device__ __forceinline__ int key(const Raw& q, int j) {
        return j == 0 ? (int)((q.t.x & 0xffffu) << 2) : j == 1 ? (int)((q.t.x >> 16) << 2)
             : j == 2 ? (int)((q.t.y & 0xffffu) << 2) : (int)((q.t.y >> 16) << 2);
    }
    // what the search remembers of entry i of a lane's quads, and the topic it stands for
    static __device__ __forceinline__ uint32_t handle(const Raw*, int i) { return (uint32_t)i; }
    template <int kQuads>
    static __device__ __forceinline__ int topic_of(const Raw* raw, uint32_t h) {
        uint32_t pair = raw[0].t.x;
#pragma unroll
        for (int p = 1; p < 2 * kQuads; ++p)
            if ((h >> 1) == (uint32_t)p) pair = (p & 1) ? raw[p / 2].t.y : raw[p / 2].t.x;
        return (int)((h & 1u) ? (pair >> 16) : (pair & 0xffffu));
    }
};

// 4 bytes per entry: uint32 entries[round4(nnz)], entry = count << 18 | topic << 2, so that the
// low 18 bits are the topic's key.  Usable when no document has 16384 tokens or more.
struct PackedRows {
    static constexpr int kEntryBytes = 4;
    static constexpr int kWavesPerSimd = 6;
    static constexpr int kMaxCount = (1 << 14) - 1;
    struct Raw {
        uint4 e;
    };
    // Every lane loads: a lane without entries reads the four padding entries that the
    // library keeps in the first 16 bytes of the slot buffer (no slot starts there).
    static __device__ __forceinline__ Raw load(const unsigned char* slots, uint32_t off, int,
                                               int e, bool on, int) {
        static_assert(kRowHeader == 16, "a row's entries start one 16-byte unit into its slot");
        uint32_t unit = on ? off + 1u + ((uint32_t)e >> 2) : 0u;
        // the choice is made on the 32-bit unit number, before it becomes a 64-bit address
        asm volatile("" : "+v"(unit));
        Raw q;
        q.e = *reinterpret_cast<const uint4*>(slots + (size_t)unit * 16u);
        return q;
    }
    static __device__ __forceinline__ uint32_t entry(const Raw& q, int j) {
        return j == 0 ? q.e.x : j == 1 ? q.e.y : j == 2 ? q.e.z : q.e.w;
    }
    static __device__ __forceinline__ int count(const Raw& q, int j) { return (int)(entry(q, j) >> 18); }
    static __device__ __forceinline__ int key(const Raw& q, int j) { return (int)(entry(q, j) & 0x3fffcu); }
    static __device__ __forceinline__ uint32_t handle(const Raw* raw, int i) {
        return entry(raw[i / 4], i % 4);
    }
    template <int kQuads>
    static __device__ __forceinline__ int topic_of(const Raw*, uint32_t h) {
        return (int)((h >> 2) & 0xffffu);
    }
};

// p*(k) is staged at the very start of the workgroup's LDS, so a topic's key (4 k) is the
// LDS address of its weight.
__device__ __forceinline__ float lds_float_at(uint32_t byte_address) {
    typedef __attribute__((address_space(3))) const float* lds_float_ptr;
    return *(lds_float_ptr)(uintptr_t)byte_address;
}

// p1 = (count - [k = o]) * p*'(k), Eq. 6, accumulated onto `base`:
// s[j] = base + p1_0 + .. + p1_j (each product is exact in fp64).
struct QuadSums {
    double s[4];
};

template <class Layout>
__device__ __forceinline__ QuadSums quad_sums(const typename Layout::Raw& raw, int o_key, float w_o,
                                              const float* pstar, double base) {
    QuadSums q;
    int key[4];
    float w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        key[j] = Layout::key(raw, j);
        w[j] = lds_float_at((uint32_t)key[j]);
    }
    double acc = base;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool own = key[j] == o_key;
        acc = fma((double)(Layout::count(raw, j) - (own ? 1 : 0)), (double)(own ? w_o : w[j]), acc);
        q.s[j] = acc;
    }
    return q;
}

// What the lanes of a group need of their token, read back from its record.
struct RowCtx {
    int o_key;              // 4 * current topic (a topic's key is its byte offset in p*)
    float w_o;
    double u, Qp;
};

__device__ __forceinline__ RowCtx row_ctx(const TokenRec* rec) {
    const int2 ow = *reinterpret_cast<const int2*>(&rec->o);
    const double2 uq = *reinterpret_cast<const double2*>(&rec->u);
    RowCtx r;
    r.o_key = ow.x << 2; r.w_o = __int_as_float(ow.y); r.u = uq.x; r.Qp = uq.y;
    return r;
}

// Row total S (Eq. 7), the draw x = u (S + Q'), and whether this lane's entries hold it.
struct RowDraw {
    double S, x, y;         // y = x - (sum of the group's sub-lanes before this one)
    bool sparse, hit;
};

template <int kLanes>
__device__ __forceinline__ RowDraw row_draw(double lane_sum, const RowCtx& r, int sl, int lane) {
    RowDraw d;
    const double incl = group_inclusive_sum<kLanes>(lane_sum);
    const double excl = group_previous<kLanes>(incl, sl);
    d.S = __shfl(incl, group_last_lane<kLanes>(lane), kWave);
    d.x = r.u * (d.S + r.Qp);
    d.sparse = d.x < d.S;
    d.hit = d.sparse && (incl > d.x) && !(excl > d.x);
    d.y = d.x - excl;
    return d;
}

// The result goes back in the token's record.  Records of a batch's unused tail take part
// like any other (their rows are empty): what is written there is never read.
__device__ __forceinline__ void row_store(TokenRec* rec, int sl, const RowDraw& d, int k_sel) {
    if (d.hit) rec->off = (uint32_t)k_sel;
    if (!d.sparse && sl == 0) {
        rec->off = 0xffffffffu;             // the draw falls into the dense bucket p2
        rec->u = d.x - d.S;
    }
}

// Rows whose sub-lanes own at most kQuads quads, already loaded: every lane keeps its prefix
// sums in registers, and the entries as loaded.
template <class Layout, int kLanes, int kQuads>
__device__ __forceinline__ void row_pass_kept(TokenRec* rec, int sl, const typename Layout::Raw* raw,
                                              const float* pstar, int lane) {
    const RowCtx r = row_ctx(rec);
    QuadSums q[kQuads];
    double acc = 0.0;
#pragma unroll
    for (int c = 0; c < kQuads; ++c) {
        q[c] = quad_sums<Layout>(raw[c], r.o_key, r.w_o, pstar, acc);
        acc = q[c].s[3];
    }
    const RowDraw d = row_draw<kLanes>(acc, r, sl, lane);
    // smallest entry whose prefix exceeds y (the prefixes never decrease)
    uint32_t sel = Layout::handle(raw, 4 * kQuads - 1);
#pragma unroll
    for (int i = 4 * kQuads - 2; i >= 0; --i)
        if (q[i / 4].s[i % 4] > d.y) sel = Layout::handle(raw, i);
    if (__ballot(d.hit && !(acc > d.y)) != 0) {      // rounding left no prefix above the draw:
        if (d.hit && !(acc > d.y)) {                 // take the lane's last entry with weight
            double before = 0.0;
#pragma unroll
            for (int i = 0; i < 4 * kQuads; ++i) {
                if (q[i / 4].s[i % 4] > before) sel = Layout::handle(raw, i);
                before = q[i / 4].s[i % 4];
            }
        }
    }
    row_store(rec, sl, d, Layout::template topic_of<kQuads>(raw, sel));
}

// Rows of more than 768 entries, one per wave (sub-lane = lane): one walk for the sums, a
// second one over the hit lane's entries.  Lane l owns the entries [4 n4 l, 4 n4 (l + 1)).
template <class Layout>
__device__ __forceinline__ void row_pass_long(const unsigned char* slots, TokenRec* rec, int K,
                                              const float* pstar, int lane) {
    const uint2 where = *reinterpret_cast<const uint2*>(rec);
    const uint32_t off = where.x;
    const int nnz = (int)where.y, n4 = (nnz + 4 * kWave - 1) / (4 * kWave);
    const RowCtx r = row_ctx(rec);
    const int e0 = lane * 4 * n4;
    double acc = 0.0;
    for (int c = 0; c < n4; ++c) {
        const int e = e0 + 4 * c;
        const QuadSums q = quad_sums<Layout>(Layout::load(slots, off, nnz, e, e < nnz, K),
                                             r.o_key, r.w_o, pstar, acc);
        acc = q.s[3];
    }
    const RowDraw d = row_draw<kWave>(acc, r, lane, lane);
    int k_sel = 0;
    if (__ballot(d.hit) != 0) {
        bool ok = false;
        int last_k = 0;
        acc = 0.0;
        for (int c = 0; c < n4; ++c) {
            const int e = e0 + 4 * c;
            const typename Layout::Raw raw = Layout::load(slots, off, nnz, e, d.hit && e < nnz, K);
            const QuadSums q = quad_sums<Layout>(raw, r.o_key, r.w_o, pstar, acc);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double before = (j == 0) ? acc : q.s[j - 1];
                if (!ok && q.s[j] > d.y) { k_sel = Layout::key(raw, j) >> 2; ok = true; }
                if (q.s[j] > before) last_k = Layout::key(raw, j) >> 2;
            }
            acc = q.s[3];
        }
        if (!ok) k_sel = last_k;
    }
    row_store(rec, lane, d, k_sel);
}

template <int kWaves, class Layout>
// Six waves per SIMD (80 VGPRs) with 4-byte entries, five (96 VGPRs) with 6-byte entries,
// whose quads take half as many registers again: the walk hides HBM latency by occupancy as
// well as by the early loads.
__attribute__((amdgpu_waves_per_eu(Layout::kWavesPerSimd)))
__global__ __launch_bounds__(kWaves * kWave) void sample_kernel(const SampleArgs a) {
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int kGroup = dense_group(kWaves);
    const int K = a.K, Kpad = a.Kpad, ng = Kpad / kGroup;
    float* pstar = reinterpret_cast<float*>(lds);
    double* cp = reinterpret_cast<double*>(lds + (size_t)Kpad * 4);
    const int tid = (int)threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);      // wave-uniform, in an SGPR
    unsigned char* wave_base = lds + (size_t)Kpad * 4 + (size_t)((ng + 1) & ~1) * 8;
    TokenRec* my_rec = reinterpret_cast<TokenRec*>(wave_base) + wave * kWave;

    Tile tl = a.tiles[blockIdx.x];         // the same for every lane: keep it in SGPRs
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

    // a pass shape's lane geometry: token of the lane relative to the pass's first, the lane's
    // place inside its group, its first quad of entries
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
        const int pos = tl.begin + idx;
        TokenRec mine;
        mine.off = 0; mine.nnz = 0; mine.o = 0; mine.w_o = 0.f; mine.u = 0.0; mine.Qp = 0.0;
        double delta = 0.0;
        if (valid) {
            mine.off = a.tok_slot[pos];
            mine.o = (int)a.z_cur[pos];
            const uint64_t id = (uint64_t)(uint32_t)a.tok_id[pos];
            // the row's length sits in front of its entries: this read also brings the row's
            // first line on its way
            mine.nnz = *reinterpret_cast<const int32_t*>(a.slots + (size_t)mine.off * 16u);
            mine.u = token_uniform(a.seed, a.iter, id);
            // the token itself is taken out of phi and n_k at its own topic
            // (its cell of phi, of either width, is cut out of the aligned dword that holds it)
            const size_t own_byte = (phi_cell0 + (size_t)mine.o) << phi_shift;
            const uint32_t own_dword = *reinterpret_cast<const uint32_t*>(phi_cells + (own_byte & ~(size_t)3));
            const int32_t phi_own = (int32_t)((own_dword >> (((uint32_t)own_byte & 2u) << 3)) & phi_mask);
            mine.w_o = (float)(((double)(phi_own - 1) + a.beta) /
                               ((double)(a.n_k[mine.o] - 1) + a.beta_V));
            delta = (double)mine.w_o - (double)pstar[mine.o];
            // cp[ng - 1] = sum_k p*(k), read from LDS where it is needed; Q = alpha sum (Eq. 7)
            mine.Qp = a.alpha * (cp[ng - 1] + delta);
        }
        my_rec[lane] = mine;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- one token per group of 4 .. 64 lanes.  A pass takes the next 16, 8, 4, 2 or 1
        // tokens, as many as lets every lane own at most kKeptQuads quads; the rows of the
        // following pass are requested from memory before this one is worked on.
        // Shapes of a pass (lanes per token, quads per lane -> entries per row at most):
        //   0 (4,1) 16   1 (4,2) 32   2 (8,2) 64   3 (8,3) 96   4 (16,2) 128   5 (16,3) 192
        //   6 (32,2) 256   7 (32,3) 384   8 (64,2) 512   9 (64,3) 768
        //   10 = one longer row, walked twice by the wave
        // Which tokens of the batch have rows beyond each of these lengths (lanes past the
        // batch's end hold nnz = 0): the shape of every pass follows from these masks.
        const int n_here = min(batch, tl.count - b * batch);
        static_assert(kKeptQuads == 3, "the pass shapes assume three kept quads per lane");
        const uint64_t over16 = __ballot(mine.nnz > 16), over32 = __ballot(mine.nnz > 32);
        const uint64_t over64 = __ballot(mine.nnz > 64), over96 = __ballot(mine.nnz > 96);
        const uint64_t over128 = __ballot(mine.nnz > 128), over192 = __ballot(mine.nnz > 192);
        const uint64_t over256 = __ballot(mine.nnz > 256), over384 = __ballot(mine.nnz > 384);
        const uint64_t over512 = __ballot(mine.nnz > 512), over768 = __ballot(mine.nnz > 768);
        auto any = [](uint64_t mask, int t0, uint32_t window) {      // 1 if a token of the window is set
            const uint32_t w = (uint32_t)(mask >> t0) & window;
            return min(1, (int)__builtin_popcount(w));      // stays scalar arithmetic
        };
        auto shape_at = [&](int t0) {
            if (!any(over32, t0, 0xffffu)) return any(over16, t0, 0xffffu);
            if (!any(over96, t0, 0xffu)) return 2 + any(over64, t0, 0xffu);
            if (!any(over192, t0, 0xfu)) return 4 + any(over128, t0, 0xfu);
            if (!any(over384, t0, 0x3u)) return 6 + any(over256, t0, 0x3u);
            if (!any(over768, t0, 0x1u)) return 8 + any(over512, t0, 0x1u);
            return 10;
        };
        auto lanes_log2 = [](int shape) { return (int)((0x66655443322ull >> (4 * shape)) & 0xfull); };
        auto quads_of = [](int shape) { return (int)((0x03232323221ull >> (4 * shape)) & 0xfull); };
        // where a pass's rows are, and the loads of the quads its lanes keep.  `rec` is the
        // record of the lane's token, `sl` the lane's place inside its group.  A pass that
        // would run past the batch's 64 records works on the last one several times over.
        using Raw = typename Layout::Raw;
        auto request = [&](int t0, int shape, TokenRec*& rec, int& sl, Raw* raw) {
            const int nq = quads_of(shape);
            if (shape != geo_shape) {       // the lanes' places change only with the shape
                const int lg = lanes_log2(shape);
                const int g = lg < 4 ? 4 - lg : 0, hs = lg < 4 ? 4 : lg;    // interleave, run length
                geo_shape = shape;
                geo_rel = ((lane >> hs) << g) | (lane & ((1 << g) - 1));
                geo_sl = (lane & ((1 << hs) - 1)) >> g;
                geo_q0 = geo_sl * nq;        // the lane's first quad
            }
            sl = geo_sl;
            rec = my_rec + min(t0 + geo_rel, kWave - 1);
            const uint2 where = *reinterpret_cast<const uint2*>(rec);
            const int nnz = (int)where.y;
            // quads the lane loads: those of the shape that the row still has from q0 on
            const int n_mine = min(((nnz + 3) >> 2) - geo_q0, nq);
#pragma unroll
            for (int c = 0; c < kKeptQuads; ++c)
                raw[c] = Layout::load(a.slots, where.x, nnz, 4 * (geo_q0 + c), c < n_mine, K);
        };
        int t_next = 0, shape_next = shape_at(0), sl_next;
        TokenRec* rec_next;
        // one pass: `mine_raw` holds its rows, already requested; the following pass's rows
        // go to `next_raw`.  The two buffers swap roles from pass to pass.
        auto pass = [&](Raw* mine_raw, Raw* next_raw) {
            const int shape = shape_next, sl = sl_next;
            TokenRec* rec = rec_next;
            t_next += kWave >> lanes_log2(shape);
            if (t_next < n_here) {
                shape_next = shape_at(t_next);
                request(t_next, shape_next, rec_next, sl_next, next_raw);
            }
            switch (shape) {
            case 0: row_pass_kept<Layout, 4, 1>(rec, sl, mine_raw, pstar, lane); break;
            case 1: row_pass_kept<Layout, 4, 2>(rec, sl, mine_raw, pstar, lane); break;
            case 2: row_pass_kept<Layout, 8, 2>(rec, sl, mine_raw, pstar, lane); break;
            case 3: row_pass_kept<Layout, 8, 3>(rec, sl, mine_raw, pstar, lane); break;
            case 4: row_pass_kept<Layout, 16, 2>(rec, sl, mine_raw, pstar, lane); break;
            case 5: row_pass_kept<Layout, 16, 3>(rec, sl, mine_raw, pstar, lane); break;
            case 6: row_pass_kept<Layout, 32, 2>(rec, sl, mine_raw, pstar, lane); break;
            case 7: row_pass_kept<Layout, 32, 3>(rec, sl, mine_raw, pstar, lane); break;
            case 8: row_pass_kept<Layout, 64, 2>(rec, sl, mine_raw, pstar, lane); break;
            case 9: row_pass_kept<Layout, 64, 3>(rec, sl, mine_raw, pstar, lane); break;
            default: row_pass_long<Layout>(a.slots, rec, K, pstar, lane); break;
            }
        };
        Raw raw_a[kKeptQuads], raw_b[kKeptQuads];
        request(0, shape_next, rec_next, sl_next, raw_a);
        while (t_next < n_here) {
            pass(raw_a, raw_b);
            if (t_next < n_here) pass(raw_b, raw_a);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- one token per lane again: dense bucket, store
        // (the token's topic and corrected weight are read back from its record rather than
        // kept in registers across the passes)
        if (lane < batch && b * batch + lane < tl.count) {
            const TokenRec* rec = &my_rec[lane];
            int z_new = (int)rec->off;
            if (z_new < 0) {
                const int o = rec->o;
                const float w_o = rec->w_o;
                z_new = dense_bucket_search<kGroup>(pstar, cp, K, ng, a.alpha, rec->u, o, w_o,
                                                    (double)w_o - (double)pstar[o]);
            }
            a.z_next[tl.begin + b * batch + lane] = (uint16_t)z_new;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
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
