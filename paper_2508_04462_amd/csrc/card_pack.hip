// Weight re-layout (canonical row-major -> matrix-instruction fragments in stream order) and the KV read-back helper.
#pragma once
#include "card_common.hip"

namespace card {

// ------------------------------------------------------------------------------------------
// Weight re-layout: canonical row-major bf16 -> fragments in stream order.  One thread per 8-element chunk.
// ------------------------------------------------------------------------------------------
enum RowMap { MAP_IDENT = 0, MAP_ROPE = 1, MAP_GATE = 2, MAP_UP = 3 };

struct PackArgs {
    const __bf16* src;  // [src_rows][K]
    __bf16* dst;        // packed matrix base
    int32_t src_rows, K, Ks, n_rows;  // n_rows: packed rows this call fills (incl. zero padding)
    int32_t Nt, NB, nwg;              // stream order: tiles of the matrix, batch width, grid size
    int32_t prow0;      // first packed row (MAP_IDENT / MAP_ROPE)
    int32_t map, head_dim;
};

__global__ __launch_bounds__(256) void k_pack(PackArgs a) {
    const int64_t chunks_per_row = int64_t(a.Ks) * 4;
    const int64_t id = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (id >= int64_t(a.n_rows) * chunks_per_row) return;
    const int idx = int(id / chunks_per_row), ch = int(id % chunks_per_row);
    int prow, srow;
    if (a.map == MAP_IDENT) {
        prow = a.prow0 + idx;
        srow = idx;
    } else if (a.map == MAP_ROPE) {
        prow = a.prow0 + idx;
        const int h = a.head_dim, i = idx % h;
        srow = (idx / h) * h + (i >> 1) + (i & 1) * (h >> 1);
    } else {
        prow = (idx >> 3) * 16 + (idx & 7) + (a.map == MAP_UP ? 8 : 0);
        srow = idx;
    }
    const int k0 = ch * 8;
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = static_cast<__bf16>(0.f);
    if (srow < a.src_rows && k0 < a.K) v = *reinterpret_cast<const bf16x8*>(a.src + size_t(srow) * a.K + k0);
    const int t = prow >> 4, s = ch >> 2;
    const int lane = (ch & 3) * 16 + (prow & 15);
    reinterpret_cast<bf16x8*>(a.dst)[size_t(stream_frag_index(a.Nt, a.Ks, a.NB, a.nwg, t, s)) * 64 + lane] = v;
}

// A workspace is prepared by clearing all of it (control words must start at zero; the kernel
// multiplies hand-over bytes it never wrote - rows beyond r, k-steps beyond a wavefront's share
// - with zero weights, so those bytes have to be finite) and setting the mark that says so.
__global__ __launch_bounds__(256) void k_ws_init(uint4v* ws, size_t n16, uint32_t* magic_word) {
    const size_t stride = size_t(gridDim.x) * 256;
    for (size_t i = size_t(blockIdx.x) * 256 + threadIdx.x; i < n16; i += stride) ws[i] = uint4v{0u, 0u, 0u, 0u};
    // the mark lives in a 16-byte unit that this same thread has just cleared
    const size_t mi = size_t(reinterpret_cast<char*>(magic_word) - reinterpret_cast<char*>(ws)) / 16;
    if (mi % stride == size_t(blockIdx.x) * 256 + threadIdx.x) *magic_word = kWsMagic;
}

// Cache construction, eqs. (3)-(7): score every (parent, top-k token) pair w = p * sigma(parent),
// pool the M * k tuples and keep the K best, best first; equal scores in (parent, rank) order.  One
// workgroup: M * k <= 256 * kSelPerThread elements, K rounds of "largest key in the workgroup".
constexpr int kSelPerThread = 8;
struct SelectArgs {
    const float* sigma;     // [M] cumulative probability of each parent sequence, eq. (4)
    const int32_t* tok;     // [M][k] eq. (2)
    const float* prob;      // [M][k]
    int32_t M, k, K;
    int32_t* out_tok;       // [K]
    float* out_score;       // [K] eq. (3)
    int32_t* out_parent;    // [K]
};

__global__ __launch_bounds__(256) void k_cache_select(SelectArgs a) {
    __shared__ unsigned long long wbest[2][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int total = a.M * a.k;
    unsigned long long mine[kSelPerThread];
#pragma unroll
    for (int e = 0; e < kSelPerThread; ++e) {
        const int flat = tid + e * 256;
        mine[e] = 0ull;
        if (flat < total && a.tok[flat] >= 0) {
            const float w = a.prob[flat] * a.sigma[flat / a.k];
            // non-negative floats order like their bit patterns; +1 keeps a zero score above "empty"
            mine[e] = ((static_cast<unsigned long long>(__float_as_uint(w)) + 1ull) << 32) | (0xffffffffu - uint32_t(flat));
        }
    }
    const int n_out = a.K < total ? a.K : total;
    for (int j = 0; j < n_out; ++j) {
        unsigned long long best = 0ull;
#pragma unroll
        for (int e = 0; e < kSelPerThread; ++e) best = mine[e] > best ? mine[e] : best;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long other = __shfl_xor(best, o);
            best = other > best ? other : best;
        }
        if (lane == 0) wbest[j & 1][wave] = best;
        __syncthreads();
        best = wbest[j & 1][0];
#pragma unroll
        for (int w = 1; w < 4; ++w) best = wbest[j & 1][w] > best ? wbest[j & 1][w] : best;
        if (best != 0ull) {
#pragma unroll
            for (int e = 0; e < kSelPerThread; ++e) mine[e] = mine[e] == best ? 0ull : mine[e];
        }
        if (tid == 0) {
            if (best != 0ull) {
                const int flat = int(0xffffffffu - uint32_t(best & 0xffffffffull));
                a.out_tok[j] = a.tok[flat];
                a.out_score[j] = __uint_as_float(uint32_t((best >> 32) - 1ull));
                a.out_parent[j] = flat / a.k;
            } else {
                a.out_tok[j] = -1;
                a.out_score[j] = 0.f;
                a.out_parent[j] = -1;
            }
        }
    }
}

struct GatherArgs {
    const __bf16* kpool;
    const __bf16* vpool;
    const int32_t* block_table;
    int32_t first, count, n_kv_heads, head_dim;
    float* k_out;
    float* v_out;
};

__global__ __launch_bounds__(256) void k_kv_gather(GatherArgs a) {
    const int64_t id = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int h = a.head_dim;
    if (id >= int64_t(a.count) * a.n_kv_heads * h) return;
    const int j = int(id % h), head = int((id / h) % a.n_kv_heads), i = int(id / (int64_t(h) * a.n_kv_heads));
    const int slot = a.first + i;
    const int page = a.block_table[slot >> 4], tk = slot & 15;
    const size_t base = (size_t(page) * a.n_kv_heads + head) * (16 * h);
    a.k_out[id] = static_cast<float>(a.kpool[base + ((j >> 3) * 16 + tk) * 8 + (j & 7)]);
    a.v_out[id] = static_cast<float>(a.vpool[base + v_page_index(j, tk)]);
}

}  // namespace card
