// Sampling kernel: one pass of the sparsity-aware sampler (paper Section 6.1, Eq. 6-8,
// Algorithm 2) over word-sorted tokens.
//
// Mapping to gfx950 (the paper's own mapping, warp = sampler with 32-way index trees,
// was made for 32-wide warps):
//   - a workgroup owns one tile = up to kTileTokens consecutive tokens of ONE word and
//     stages that word's p*(k) (Eq. 8) once in LDS as fp32, with fp64 prefix sums over
//     groups of 16 topics (Section 6.1.2: samplers of a block share the word's data);
//   - each wave takes 64 tokens at a time.  Everything that is per token and needs no
//     cooperation is done one token per LANE: the Philox uniform, the token's own-count
//     correction of p*(o), and the search in the dense bucket p2;
//   - the walk over the token's sparse theta row (S and the p1 prefix sums, Eq. 6-7) is
//     done one token per WAVE with coalesced loads of the row and an fp64 wave scan; the
//     "smallest k whose prefix exceeds the draw" search (Section 6.1.1) is a ballot.
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
    const unsigned char* slots; // theta rows: int32 counts[round4(nnz)] then uint16 topics[round4(nnz)]
    const int32_t* n_wk;        // [V][K]
    const int32_t* n_k;         // [K]
    int32_t K, Kpad;            // Kpad = K rounded up to 16
    double alpha, beta, beta_V;
    uint64_t seed;
    uint32_t iter;
};

constexpr int kGroup = 16;      // topics per fp64 prefix group of the dense bucket

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

template <int kWaves>
__global__ __launch_bounds__(kWaves * kWave) void sample_kernel(const SampleArgs a) {
    extern __shared__ __align__(16) unsigned char lds[];
    float* pstar = reinterpret_cast<float*>(lds);
    const int K = a.K, Kpad = a.Kpad, ng = Kpad / kGroup;
    double* cp = reinterpret_cast<double*>(lds + (size_t)Kpad * sizeof(float));

    const Tile tl = a.tiles[blockIdx.x];
    const int tid = (int)threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
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

    const int n_batches = (tl.count + kWave - 1) / kWave;
    for (int b = wave; b < n_batches; b += kWaves) {
        // ---- one token per lane: token, uniform, own-count correction
        const int idx = b * kWave + lane;
        const bool valid = idx < tl.count;
        const int pos = tl.begin + idx;
        int o = 0, nnz = 0, off = 0;
        float w_o = 0.f;
        double u = 0.0, Qp = 0.0, delta = 0.0;
        if (valid) {
            const int d = a.tok_doc[pos];
            o = (int)a.z_cur[pos];
            const uint64_t id = (uint64_t)(uint32_t)a.tok_id[pos];
            const uint2 rec = a.row_rec[d];
            off = (int)rec.x;
            nnz = (int)rec.y;
            u = token_uniform(a.seed, a.iter, id);
            // the token itself is taken out of phi and n_k at its own topic
            w_o = (float)(((double)(phi_v[o] - 1) + a.beta) / ((double)(a.n_k[o] - 1) + a.beta_V));
            delta = (double)w_o - (double)pstar[o];
            Qp = a.alpha * (W + delta);
        }
        double S_mine = 0.0;
        int z_new = -1;                    // -1: the draw falls into the dense bucket

        // ---- one token per wave: sparse row of theta, S, and the p1 bucket
        const int n_here = min(kWave, tl.count - b * kWave);
        for (int i = 0; i < n_here; ++i) {
            const int nnz_i = read_lane(nnz, i);
            const int o_i = read_lane(o, i);
            const float w_o_i = read_lane(w_o, i);
            const double u_i = read_lane(u, i);
            const double Qp_i = read_lane(Qp, i);
            const int32_t* cnt = reinterpret_cast<const int32_t*>(
                a.slots + (size_t)(uint32_t)read_lane(off, i) * 16u);
            const uint16_t* top = reinterpret_cast<const uint16_t*>(cnt + ((nnz_i + 3) & ~3));
            double S;
            int z_sparse = -1;
            if (nnz_i <= kWave) {
                const bool have = lane < nnz_i;
                int c = 0, k = 0;
                if (have) { c = cnt[lane]; k = (int)top[lane]; }
                float w = pstar[k];
                if (have && k == o_i) { c -= 1; w = w_o_i; }
                const double p1 = (double)c * (double)w;            // Eq. 6, exact product
                const double incl = wave_inclusive_sum(p1);
                S = read_lane(incl, kWave - 1);
                const double x = u_i * (S + Qp_i);
                if (x < S) {
                    uint64_t m = __ballot(incl > x);
                    int j;
                    if (m != 0) j = __ffsll((unsigned long long)m) - 1;
                    else j = 63 - __clzll((unsigned long long)__ballot(p1 > 0.0));
                    z_sparse = read_lane(k, j);
                }
            } else {
                double acc = 0.0;
                for (int base = 0; base < nnz_i; base += kWave) {
                    const int j = base + lane;
                    const bool have = j < nnz_i;
                    int c = 0, k = 0;
                    if (have) { c = cnt[j]; k = (int)top[j]; }
                    float w = pstar[k];
                    if (have && k == o_i) { c -= 1; w = w_o_i; }
                    acc += (double)c * (double)w;
                }
                S = wave_sum(acc);
                const double x = u_i * (S + Qp_i);
                if (x < S) {
                    double carry = 0.0;
                    int last_k = 0;
                    for (int base = 0; base < nnz_i; base += kWave) {
                        const int j = base + lane;
                        const bool have = j < nnz_i;
                        int c = 0, k = 0;
                        if (have) { c = cnt[j]; k = (int)top[j]; }
                        float w = pstar[k];
                        if (have && k == o_i) { c -= 1; w = w_o_i; }
                        const double p1 = (double)c * (double)w;
                        const double incl = wave_inclusive_sum(p1) + carry;
                        const uint64_t m = __ballot(incl > x);
                        if (m != 0) {
                            z_sparse = read_lane(k, __ffsll((unsigned long long)m) - 1);
                            break;
                        }
                        const uint64_t mp = __ballot(p1 > 0.0);
                        if (mp != 0) last_k = read_lane(k, 63 - __clzll((unsigned long long)mp));
                        carry = read_lane(incl, kWave - 1);
                    }
                    if (z_sparse < 0) z_sparse = last_k;   // rounding left no prefix above x
                }
            }
            if (lane == i) { S_mine = S; z_new = z_sparse; }
        }

        // ---- one token per lane again: dense bucket, store
        if (valid) {
            if (z_new < 0) {
                const double x = u * (S_mine + Qp);
                z_new = dense_bucket_search(pstar, cp, K, ng, a.alpha, x - S_mine, o, w_o, delta);
            }
            a.z_next[pos] = (uint16_t)z_new;
        }
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
