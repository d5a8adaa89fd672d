// Sampling kernel: one pass of the sparsity-aware sampler (paper Section 6.1, Eq. 6-8,
// Algorithm 2) over word-sorted tokens.
//
// Mapping to gfx950 (the paper's own mapping, one 32-wide warp per sampler with 32-way
// index trees, was made for NVIDIA warps; measured here, a whole 64-lane wave per token is
// bound by VALU issue, not by HBM):
//   - a workgroup owns one tile = up to 1024 (4096 for large K) consecutive tokens of ONE
//     word and stages that word's p*(k) (Eq. 8) once in LDS as fp32, with fp64 prefix sums
//     over groups of 16 topics (Section 6.1.2: samplers of a block share the word's data);
//   - each wave takes 64 tokens at a time.  What is per token and needs no cooperation is
//     done one token per LANE: the Philox uniform, the token's own-count correction of
//     p*(o), and the search in the dense bucket p2 (binary search over the group prefixes,
//     then at most 16 steps);
//   - the walk over the token's sparse theta row (S and the p1 prefix sums, Eq. 6-7) is done
//     by 16 lanes per token (one DPP row), four tokens per wave at a time: every lane owns
//     a contiguous run of entries, loaded four at a time as one 16-byte and one 8-byte
//     load, accumulates them in fp64, and a 4-step in-row DPP scan gives the prefix over
//     lanes.  The lane whose range holds the draw finds "the smallest k whose prefix exceeds
//     it" (Section 6.1.1) among its own entries.  Token parameters and results travel
//     between the per-lane and per-row phases through small per-wave LDS records;
//   - the row walk is a chain of dependent loads (record, then a random row in HBM), so the
//     loads of the next four rows are issued before the current four are worked on.
#pragma once
#include "device_util.hpp"

namespace mlda {

struct Tile {          // consecutive word-major tokens of one word
    int32_t word;
    int32_t begin;     // first word-major token position
    int32_t count;     // 1 .. tile size
    int32_t whole;     // 1 if the tile holds every token of its word
};

struct SampleArgs {
    const Tile* tiles;
    const int32_t* tok_doc;     // [T] document of each word-major token
    const int32_t* tok_id;      // [T] its index in the caller's document-major order
    const uint16_t* z_cur;      // [T] word-major, frozen for the pass
    uint16_t* z_next;           // [T] word-major, written
    const uint2* row_rec;       // [D] {slot offset in 16-byte units, nnz of the theta row}
    // theta rows: int32 counts[round4(nnz)] then uint16 topics[round4(nnz)]; padding entries
    // hold count 0 and topic K
    const unsigned char* slots;
    const int32_t* n_wk;        // [V][K]
    const int32_t* n_k;         // [K]
    int32_t K, Kpad;            // Kpad = K+1 rounded up to 16: p*(K..Kpad-1) = 0
    double alpha, beta, beta_V;
    uint64_t seed;
    uint32_t iter;
};

constexpr int kGroup = 16;      // topics per fp64 prefix group of the dense bucket
constexpr int kRowLanes = 16;   // lanes that walk one token's theta row (one DPP row)
constexpr int kRowsPerWave = kWave / kRowLanes;
constexpr int kAheadQuads = 2;  // quads per lane whose loads are issued one pass ahead

struct __align__(16) TokenRec { // per-lane phase -> per-row phase, 32 bytes
    uint32_t off;               // slot offset of the token's theta row, 16-byte units
    int32_t nnz;
    int32_t o;                  // current topic
    float w_o;                  // p*(o) with the token itself removed
    double u;
    double Qp;                  // alpha * sum_k p*'(k)
};

// LDS bytes of sample_kernel<kWaves> for a given Kpad.
__host__ __device__ constexpr size_t sample_lds_bytes(int Kpad, int waves) {
    return (size_t)Kpad * 4 + (size_t)((Kpad / kGroup + 1) & ~1) * 8 +
           (size_t)waves * kWave * (8 + sizeof(TokenRec) + 4);
}

// Dense bucket (p2 = alpha p*', Eq. 6): smallest k with alpha * prefix'(k) > y, where
// prefix' is the prefix sum of p* with the entry of the token's own topic o replaced by
// w_o (delta = w_o - p*(o)).  One lane per token.
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
    double acc = (lo > 0 ? cp[lo - 1] : 0.0) + (k0 > o ? delta : 0.0);
    int found = min(k0 + kGroup - 1, K - 1);
    for (int j = 0; j < kGroup; ++j) {
        const int k = k0 + j;
        if (k >= K) break;
        acc += (double)((k == o) ? w_o : pstar[k]);
        if (alpha * acc > y) { found = k; break; }
    }
    return found;
}

// Move within each row of 16 lanes; lanes without a source read 0.
template <int kCtrl>
__device__ __forceinline__ double row_move0(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), kCtrl, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), kCtrl, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

// Inclusive prefix sum inside each row of 16 lanes.  Every lane must be active.
__device__ __forceinline__ double row_inclusive_sum(double v) {
    v += row_move0<0x111>(v);   // row_shr:1
    v += row_move0<0x112>(v);   // row_shr:2
    v += row_move0<0x114>(v);   // row_shr:4
    v += row_move0<0x118>(v);   // row_shr:8
    return v;
}

// What the 16 lanes of a row need of their token.
struct RowCtx {
    uint32_t off;           // slot of the theta row, 16-byte units
    int nnz, n4;            // n4 = quads each lane owns; lane sl owns entries [4 n4 sl, 4 n4 (sl+1))
    int o;
    float w_o;
    double u, Qp;
    bool row_on;
    int ti;                 // token index inside the wave's batch
};

__device__ __forceinline__ const int32_t* row_counts(const unsigned char* slots, const RowCtx& r) {
    return reinterpret_cast<const int32_t*>(slots + (size_t)r.off * 16u);
}
__device__ __forceinline__ const uint16_t* row_topics(const unsigned char* slots, const RowCtx& r) {
    return reinterpret_cast<const uint16_t*>(row_counts(slots, r) + ((r.nnz + 3) & ~3));
}

// Four consecutive entries of a row as they come from memory.
struct QuadRaw {
    int4 c;                 // counts
    uint2 t;                // topics, two per dword
};

__device__ __forceinline__ QuadRaw quad_load(const unsigned char* slots, const RowCtx& r, int e,
                                             bool on, int K) {
    QuadRaw q;
    q.c = make_int4(0, 0, 0, 0);
    q.t = make_uint2((uint32_t)K | ((uint32_t)K << 16), (uint32_t)K | ((uint32_t)K << 16));
    if (on) {
        q.c = *reinterpret_cast<const int4*>(row_counts(slots, r) + e);
        q.t = *reinterpret_cast<const uint2*>(row_topics(slots, r) + e);
    }
    return q;
}

// p1 = (count - [k = o]) * p*'(k), Eq. 6, accumulated onto `base`:
// s[j] = base + p1_0 + .. + p1_j (each product is exact in fp64).
struct Quad {
    int k[4];
    double s[4];
};

__device__ __forceinline__ Quad quad_sums(const QuadRaw& raw, int o, float w_o, const float* pstar,
                                          double base) {
    Quad q;
    q.k[0] = (int)(raw.t.x & 0xffffu); q.k[1] = (int)(raw.t.x >> 16);
    q.k[2] = (int)(raw.t.y & 0xffffu); q.k[3] = (int)(raw.t.y >> 16);
    const int cc[4] = {raw.c.x, raw.c.y, raw.c.z, raw.c.w};
    double acc = base;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool own = q.k[j] == o;
        const float w = own ? w_o : pstar[q.k[j]];
        acc = fma((double)(cc[j] - (own ? 1 : 0)), (double)w, acc);
        q.s[j] = acc;
    }
    return q;
}

// Row total S (Eq. 7), the draw x = u (S + Q'), and whether this lane's entries hold it.
struct RowDraw {
    double S, x, y;         // y = x - (sum of the lanes before this one)
    bool sparse, hit;
};

__device__ __forceinline__ RowDraw row_draw(double lane_sum, const RowCtx& r, int lane) {
    RowDraw d;
    const double incl = row_inclusive_sum(lane_sum);
    const double excl = row_move0<0x111>(incl);
    d.S = __shfl(incl, lane | (kRowLanes - 1), kWave);
    d.x = r.u * (d.S + r.Qp);
    d.sparse = d.x < d.S;
    d.hit = d.sparse && (incl > d.x) && !(excl > d.x);
    d.y = d.x - excl;
    return d;
}

__device__ __forceinline__ void row_store(const RowCtx& r, const RowDraw& d, int k_sel, int sl,
                                          int* my_res, double* my_y) {
    if (d.hit) my_res[r.ti] = k_sel;
    if (r.row_on && !d.sparse && sl == 0) {
        my_res[r.ti] = -1;                  // the draw falls into the dense bucket p2
        my_y[r.ti] = d.x - d.S;
    }
}

// Rows of at most 64 kQuads entries, already loaded: every lane keeps its prefix sums in
// registers.
template <int kQuads>
__device__ __forceinline__ void row_pass_kept(const RowCtx& r, const QuadRaw* raw, const float* pstar,
                                              int sl, int lane, int* my_res, double* my_y) {
    Quad q[kQuads];
    double acc = 0.0;
#pragma unroll
    for (int c = 0; c < kQuads; ++c) {
        q[c] = quad_sums(raw[c], r.o, r.w_o, pstar, acc);
        acc = q[c].s[3];
    }
    const RowDraw d = row_draw(acc, r, lane);
    // smallest entry whose prefix exceeds y (the prefixes never decrease)
    int k_sel = q[kQuads - 1].k[3];
#pragma unroll
    for (int i = 4 * kQuads - 2; i >= 0; --i)
        if (q[i / 4].s[i % 4] > d.y) k_sel = q[i / 4].k[i % 4];
    if (__ballot(d.hit && !(acc > d.y)) != 0) {      // rounding left no prefix above the draw:
        if (d.hit && !(acc > d.y)) {                 // take the lane's last entry with weight
            double before = 0.0;
#pragma unroll
            for (int i = 0; i < 4 * kQuads; ++i) {
                if (q[i / 4].s[i % 4] > before) k_sel = q[i / 4].k[i % 4];
                before = q[i / 4].s[i % 4];
            }
        }
    }
    row_store(r, d, k_sel, sl, my_res, my_y);
}

// Longer rows: one walk for the sums, a second one over the hit lane's entries.
__device__ __forceinline__ void row_pass_long(const unsigned char* slots, const RowCtx& r, int n4max,
                                              int K, const float* pstar, int sl, int lane,
                                              int* my_res, double* my_y) {
    const int e0 = sl * 4 * r.n4;
    double acc = 0.0;
    for (int c = 0; c < n4max; ++c) {
        const int e = e0 + 4 * c;
        const Quad q = quad_sums(quad_load(slots, r, e, c < r.n4 && e < r.nnz, K), r.o, r.w_o, pstar, acc);
        acc = q.s[3];
    }
    const RowDraw d = row_draw(acc, r, lane);
    int k_sel = 0;
    if (__ballot(d.hit) != 0) {
        bool ok = false;
        int last_k = 0;
        acc = 0.0;
        for (int c = 0; c < n4max; ++c) {
            const int e = e0 + 4 * c;
            const Quad q = quad_sums(quad_load(slots, r, e, d.hit && c < r.n4 && e < r.nnz, K), r.o,
                                     r.w_o, pstar, acc);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double before = (j == 0) ? acc : q.s[j - 1];
                if (!ok && q.s[j] > d.y) { k_sel = q.k[j]; ok = true; }
                if (q.s[j] > before) last_k = q.k[j];
            }
            acc = q.s[3];
        }
        if (!ok) k_sel = last_k;
    }
    row_store(r, d, k_sel, sl, my_res, my_y);
}

template <int kWaves>
__global__ __launch_bounds__(kWaves * kWave) void sample_kernel(const SampleArgs a) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int K = a.K, Kpad = a.Kpad, ng = Kpad / kGroup;
    float* pstar = reinterpret_cast<float*>(lds);
    double* cp = reinterpret_cast<double*>(lds + (size_t)Kpad * 4);
    const int tid = (int)threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    unsigned char* wave_base = lds + (size_t)Kpad * 4 + (size_t)((ng + 1) & ~1) * 8;
    double* my_y = reinterpret_cast<double*>(wave_base) + wave * kWave;
    TokenRec* my_rec = reinterpret_cast<TokenRec*>(wave_base + (size_t)kWaves * kWave * 8) + wave * kWave;
    int* my_res = reinterpret_cast<int*>(wave_base + (size_t)kWaves * kWave * (8 + sizeof(TokenRec))) +
                  wave * kWave;

    const Tile tl = a.tiles[blockIdx.x];
    const int32_t* phi_v = a.n_wk + (size_t)tl.word * (size_t)K;

    // ---- stage p*(k) = (phi_kv + beta)/(n_k + beta V) as fp32 (Eq. 8)
    for (int k = tid; k < Kpad; k += kWaves * kWave) {
        float w = 0.f;
        if (k < K) w = (float)(((double)phi_v[k] + a.beta) / ((double)a.n_k[k] + a.beta_V));
        pstar[k] = w;
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
    const double W = cp[ng - 1];           // sum_k p*(k);  Q = alpha W (Eq. 7)

    const int sl = lane & (kRowLanes - 1), row = lane / kRowLanes;
    const int n_batches = (tl.count + kWave - 1) / kWave;
    for (int b = wave; b < n_batches; b += kWaves) {
        // ---- one token per lane: token, uniform, own-count correction
        const int idx = b * kWave + lane;
        const bool valid = idx < tl.count;
        const int pos = tl.begin + idx;
        TokenRec mine;
        mine.off = 0; mine.nnz = 0; mine.o = 0; mine.w_o = 0.f; mine.u = 0.0; mine.Qp = 0.0;
        double delta = 0.0;
        if (valid) {
            const int d = a.tok_doc[pos];
            mine.o = (int)a.z_cur[pos];
            const uint64_t id = (uint64_t)(uint32_t)a.tok_id[pos];
            const uint2 rec = a.row_rec[d];
            mine.off = rec.x;
            mine.nnz = (int)rec.y;
            mine.u = token_uniform(a.seed, a.iter, id);
            // the token itself is taken out of phi and n_k at its own topic
            mine.w_o = (float)(((double)(phi_v[mine.o] - 1) + a.beta) /
                               ((double)(a.n_k[mine.o] - 1) + a.beta_V));
            delta = (double)mine.w_o - (double)pstar[mine.o];
            mine.Qp = a.alpha * (W + delta);
        }
        my_rec[lane] = mine;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- one token per row of 16 lanes, four tokens per pass; the rows of pass p+1 are
        // requested from memory before pass p is worked on
        const int n_here = min(kWave, tl.count - b * kWave);
        const int n_pass = (n_here + kRowsPerWave - 1) / kRowsPerWave;
        auto row_ctx = [&](int p) {
            RowCtx r;
            r.ti = p * kRowsPerWave + row;
            r.row_on = r.ti < n_here;
            const TokenRec rec = my_rec[r.row_on ? r.ti : 0];
            r.off = rec.off;
            r.nnz = r.row_on ? rec.nnz : 0;
            r.n4 = (r.nnz + 4 * kRowLanes - 1) / (4 * kRowLanes);
            r.o = rec.o; r.w_o = rec.w_o; r.u = rec.u; r.Qp = rec.Qp;
            return r;
        };
        auto longest = [&](const RowCtx& r) {          // quads per lane of the pass's longest row
            return max(max(read_lane(r.n4, 0), read_lane(r.n4, 16)),
                       max(read_lane(r.n4, 32), read_lane(r.n4, 48)));
        };
        auto request = [&](const RowCtx& r, int n4max, QuadRaw* raw) {
            const bool kept = n4max <= kAheadQuads;    // longer rows are loaded by their own walk
#pragma unroll
            for (int c = 0; c < kAheadQuads; ++c) {
                const int e = sl * 4 * r.n4 + 4 * c;
                raw[c] = quad_load(a.slots, r, e, kept && c < r.n4 && e < r.nnz, K);
            }
        };
        RowCtx r_next = row_ctx(0);
        int n4max_next = longest(r_next);
        QuadRaw raw_next[kAheadQuads];
        request(r_next, n4max_next, raw_next);
        for (int p = 0; p < n_pass; ++p) {
            const RowCtx r = r_next;
            const int n4max = n4max_next;
            QuadRaw raw[kAheadQuads];
#pragma unroll
            for (int c = 0; c < kAheadQuads; ++c) raw[c] = raw_next[c];
            if (p + 1 < n_pass) {
                r_next = row_ctx(p + 1);
                n4max_next = longest(r_next);
                request(r_next, n4max_next, raw_next);
            }
            if (n4max <= 1)      row_pass_kept<1>(r, raw, pstar, sl, lane, my_res, my_y);
            else if (n4max <= 2) row_pass_kept<2>(r, raw, pstar, sl, lane, my_res, my_y);
            else                 row_pass_long(a.slots, r, n4max, K, pstar, sl, lane, my_res, my_y);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- one token per lane again: dense bucket, store
        if (valid) {
            int z_new = my_res[lane];
            if (z_new < 0)
                z_new = dense_bucket_search(pstar, cp, K, ng, a.alpha, my_y[lane], mine.o, mine.w_o,
                                            delta);
            a.z_next[pos] = (uint16_t)z_new;
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
