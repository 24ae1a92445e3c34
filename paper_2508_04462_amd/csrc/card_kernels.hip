// Device code of the CARD verification step for gfx950 (CDNA4, 64-wide wavefronts).
//
// One step = embed -> per layer { QKV GEMM (+norm, rotation, KV write) -> chain attention over
// the paged KV cache -> O GEMM (+residual) -> gate/up GEMM (+norm, SwiGLU) -> down GEMM
// (+residual) } -> vocabulary GEMM (+norm, arg-max) -> prefix accept / correction token
// (overview figure, steps 1-3; Cache Correction).  With r <= 32 rows every GEMM reads each
// weight byte once and does r multiply-adds per element: HBM-bound.  The kernels therefore
// stream weights that were re-laid at load time into matrix-instruction register order (one
// fully contiguous 1 KiB load per wavefront and 16x32 tile), keep the r activations in fp32
// and feed them to the bf16 matrix instruction as a high + low bf16 pair (two instructions per
// tile; the matrix pipe is ~95 % idle anyway), and accumulate in fp32.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "card_layout.h"

namespace card {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(4))) float floatx4;

enum Epilogue { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3 };

struct GemmArgs {
    const bf16x8* w;      // packed matrix, tile order
    int32_t N, K, Nt, Ks; // logical rows / columns, tiles / k-steps
    int32_t splits, steps_per_split;
    const float* xin;     // [r][ldx] fp32 activations
    int32_t ldx;
    int32_t r;
    const float* gain;    // per-column gain of the preceding RMSNorm, or nullptr
    const float* ss_in;   // [ss_in_groups][32] partial sums of squares of xin rows, or nullptr
    int32_t ss_in_groups;
    float inv_d, eps;
    float* part;          // split-K partials [group][split][64][16*MT]
    int32_t* counters;    // one per group, zero on entry, zero on exit
    // epilogue outputs
    float* x;             // RESID: residual stream [r][N], updated in place
    float* ss_out;        // RESID: [groups][32] partial sums of squares of the new x
    float* q;             // QKV: [r][q_dim] rotated queries
    __bf16* kpool;        // QKV: K page pool base of this layer
    __bf16* vpool;
    const int32_t* block_table;
    const float* rope;    // cos[32][h/2], sin[32][h/2]
    int32_t ctx_len, head_dim, q_dim, kv_dim, n_kv_heads;
    float* act;           // SWIGLU: [r][F]
    int32_t F;
    unsigned long long* best;  // LMHEAD: [32] packed (logit key, ~index), zero on entry
    float* logits;        // LMHEAD debug: [r][N] or nullptr
};

// Data handed from one workgroup to another inside a kernel goes through agent-scope relaxed
// atomics: the store writes through the compute die's own L2, the load bypasses it.  That is
// enough for the "last workgroup to arrive merges" hand-off and costs far less than a full
// device fence (which writes back and invalidates the whole L2 on every call).
__device__ __forceinline__ void st_agent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// all of this thread's earlier stores have been acknowledged
__device__ __forceinline__ void wait_stores() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
}
// order-preserving map float -> uint32 (larger float, larger key)
__device__ __forceinline__ uint32_t float_key(float v) {
    const uint32_t b = __float_as_uint(v);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ void split_bf16(float v, __bf16& hi, __bf16& lo) {
    hi = static_cast<__bf16>(v);
    lo = static_cast<__bf16>(v - static_cast<float>(hi));
}

// ------------------------------------------------------------------------------------------
// Weight-streaming GEMM: out[m][n] = sum_k xin[m][k] * gain[k] * W[n][k], m < r <= 16*MT.
// Task = (group of 4 n-tiles) x (one cut of K).  The wavefronts of a workgroup take
// consecutive k-steps of the cut; their accumulators meet in LDS in a fixed order, cuts meet
// through global partials summed in cut order by whichever workgroup arrives last.
// ------------------------------------------------------------------------------------------
template <int MT, int EPI>
__global__ __launch_bounds__(kGemmWaves * 64) void k_gemm(GemmArgs a) {
    constexpr int NT = kGroupTiles;
    constexpr int COLS = 16 * MT;
    constexpr int TILE_FLOATS = NT * MT * 256;
    __shared__ float red[kGemmWaves * TILE_FLOATS];
    __shared__ float tile[TILE_FLOATS];  // [64 rows][COLS]
    __shared__ float row_scale[kMaxR];
    __shared__ int is_last;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int group = blockIdx.x / a.splits, split = blockIdx.x % a.splits;

    if (EPI != EPI_RESID) {
        // eight lanes per row add the per-group sums of squares (fixed order), then a butterfly
        const int mrow = tid >> 3, sub = tid & 7;
        float ss = 0.f;
        if (mrow < a.r)
            for (int g = sub; g < a.ss_in_groups; g += 8) ss += a.ss_in[g * kMaxR + mrow];
        ss += __shfl_xor(ss, 1);
        ss += __shfl_xor(ss, 2);
        ss += __shfl_xor(ss, 4);
        if (sub == 0 && mrow < a.r) row_scale[mrow] = 1.0f / sqrtf(ss * a.inv_d + a.eps);
    }

    const int ks0 = split * a.steps_per_split;
    const int ks1 = min(a.Ks, ks0 + a.steps_per_split);
    const int per = (ks1 - ks0 + kGemmWaves - 1) / kGemmWaves;
    const int ws0 = ks0 + wave * per;
    const int ws1 = min(ks1, ws0 + per);

    floatx4 acc[NT][MT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    const bf16x8* wt[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        int t = group * NT + i;
        if (t >= a.Nt) t = a.Nt - 1;  // results of an out-of-range tile are dropped in the epilogue
        wt[i] = a.w + size_t(t) * a.Ks * 64 + lane;
    }
    const int m = lane & 15, kc = lane >> 4;

    constexpr int U = 2;
    for (int s = ws0; s < ws1; s += U) {
        bf16x8 af[U][NT];
        float xv[U][MT][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int su = min(s + u, ws1 - 1);
#pragma unroll
            for (int i = 0; i < NT; ++i) af[u][i] = __builtin_nontemporal_load(wt[i] + size_t(su) * 64);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k0 = (s + u) * kTileK + kc * 8;
            const bool kin = (s + u) < ws1 && k0 < a.K;
            float gv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) gv[e] = 1.f;
            if (a.gain && kin) {
                const float4 g0 = *reinterpret_cast<const float4*>(a.gain + k0);
                const float4 g1 = *reinterpret_cast<const float4*>(a.gain + k0 + 4);
                gv[0] = g0.x; gv[1] = g0.y; gv[2] = g0.z; gv[3] = g0.w;
                gv[4] = g1.x; gv[5] = g1.y; gv[6] = g1.z; gv[7] = g1.w;
            }
#pragma unroll
            for (int j = 0; j < MT; ++j) {
                const int row = j * 16 + m;
                if (kin && row < a.r) {
                    const float* xp = a.xin + size_t(row) * a.ldx + k0;
                    const float4 v0 = *reinterpret_cast<const float4*>(xp);
                    const float4 v1 = *reinterpret_cast<const float4*>(xp + 4);
                    xv[u][j][0] = v0.x * gv[0]; xv[u][j][1] = v0.y * gv[1];
                    xv[u][j][2] = v0.z * gv[2]; xv[u][j][3] = v0.w * gv[3];
                    xv[u][j][4] = v1.x * gv[4]; xv[u][j][5] = v1.y * gv[5];
                    xv[u][j][6] = v1.z * gv[6]; xv[u][j][7] = v1.w * gv[7];
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) xv[u][j][e] = 0.f;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int j = 0; j < MT; ++j) {
                bf16x8 bh, bl;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    __bf16 hi, lo;
                    split_bf16(xv[u][j][e], hi, lo);
                    bh[e] = hi;
                    bl[e] = lo;
                }
#pragma unroll
                for (int i = 0; i < NT; ++i) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[u][i], bh, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[u][i], bl, acc[i][j], 0, 0, 0);
                }
            }
        }
    }

    // wavefront accumulators -> LDS, then a fixed-order sum over wavefronts
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j)
            *reinterpret_cast<floatx4*>(&red[wave * TILE_FLOATS + (i * MT + j) * 256 + lane * 4]) = acc[i][j];
    __syncthreads();
    for (int e = tid; e < TILE_FLOATS; e += kGemmWaves * 64) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kGemmWaves; ++w) s += red[w * TILE_FLOATS + e];
        const int t = e >> 8, l = (e & 255) >> 2, v = e & 3;
        const int i = t / MT, j = t % MT;
        const int nl = i * 16 + (l >> 4) * 4 + v, mm = j * 16 + (l & 15);
        tile[nl * COLS + mm] = s;
    }
    __syncthreads();

    if (a.splits > 1) {
        float* mine = a.part + (size_t(group) * a.splits + split) * (kGroupRows * COLS);
        for (int e = tid; e < kGroupRows * COLS; e += kGemmWaves * 64) st_agent(mine + e, tile[e]);
        wait_stores();
        __syncthreads();
        if (tid == 0) {
            const int prev = __hip_atomic_fetch_add(&a.counters[group], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            is_last = (prev == a.splits - 1);
        }
        __syncthreads();
        if (!is_last) return;
        const float* base = a.part + size_t(group) * a.splits * (kGroupRows * COLS);
        for (int e = tid; e < kGroupRows * COLS; e += kGemmWaves * 64) {
            float pv[kMaxSplits];
#pragma unroll
            for (int sp = 0; sp < kMaxSplits; ++sp)
                pv[sp] = sp < a.splits ? ld_agent(base + size_t(sp) * (kGroupRows * COLS) + e) : 0.f;
            float s = 0.f;
#pragma unroll
            for (int sp = 0; sp < kMaxSplits; ++sp) s += pv[sp];
            tile[e] = s;
        }
        if (tid == 0) __hip_atomic_store(&a.counters[group], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
    }

    const int r = a.r;
    const int row0 = group * kGroupRows;  // first packed row of this group
    if (EPI == EPI_RESID) {
        for (int e = tid; e < kGroupRows * r; e += kGemmWaves * 64) {
            const int nl = e % kGroupRows, mm = e / kGroupRows;
            const int n = row0 + nl;
            float nv = 0.f;
            if (n < a.N) {
                nv = a.x[size_t(mm) * a.N + n] + tile[nl * COLS + mm];
                a.x[size_t(mm) * a.N + n] = nv;
            }
            tile[nl * COLS + mm] = nv;
        }
        __syncthreads();
        if (tid < r) {
            float ss = 0.f;
            for (int nl = 0; nl < kGroupRows; ++nl) {
                const float v = tile[nl * COLS + tid];
                ss += v * v;
            }
            a.ss_out[group * kMaxR + tid] = ss;
        }
    } else if (EPI == EPI_SWIGLU) {
        // tile rows: per n-tile, rows 0..7 gate and rows 8..15 up of the same 8 FFN columns
        for (int e = tid; e < 32 * r; e += kGemmWaves * 64) {
            const int fl = e % 32, mm = e / 32;
            const int i = fl >> 3, c = fl & 7;
            const int f = (group * NT + i) * 8 + c;
            if (f < a.F) {
                const float sc = row_scale[mm];
                const float g = tile[(i * 16 + c) * COLS + mm] * sc;
                const float u = tile[(i * 16 + 8 + c) * COLS + mm] * sc;
                a.act[size_t(mm) * a.F + f] = g / (1.f + expf(-g)) * u;
            }
        }
    } else if (EPI == EPI_LMHEAD) {
        if (a.logits) {
            for (int e = tid; e < kGroupRows * r; e += kGemmWaves * 64) {
                const int nl = e % kGroupRows, mm = e / kGroupRows;
                if (row0 + nl < a.N) a.logits[size_t(mm) * a.N + row0 + nl] = tile[nl * COLS + mm] * row_scale[mm];
            }
        }
        if (tid < r) {
            const float sc = row_scale[tid];
            float best = -INFINITY;
            int bi = 0x7fffffff;
            for (int nl = 0; nl < kGroupRows; ++nl) {
                if (row0 + nl >= a.N) break;
                const float v = tile[nl * COLS + tid] * sc;
                if (v > best) {
                    best = v;
                    bi = row0 + nl;
                }
            }
            // (value, lowest index) as one 64-bit key; the maximum does not depend on arrival order
            const unsigned long long key =
                (static_cast<unsigned long long>(float_key(best)) << 32) | (0xffffffffu - uint32_t(bi));
            __hip_atomic_fetch_max(&a.best[tid], key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    } else {  // EPI_QKV
        // packed rows: [q heads | k heads | v heads]; inside a q or k head row 2p holds element p
        // of the head and row 2p+1 its rotation partner p + h/2
        const int h = a.head_dim, half = h >> 1;
        if (row0 < a.q_dim + a.kv_dim) {
            const bool is_q = row0 < a.q_dim;
            for (int e = tid; e < 32 * r; e += kGemmWaves * 64) {
                const int pl = e % 32, mm = e / 32;
                const int prow = row0 + 2 * pl;
                const int rel = is_q ? prow : prow - a.q_dim;
                const int head = rel / h, p = (rel % h) >> 1;
                const float sc = row_scale[mm];
                const float z0 = tile[(2 * pl) * COLS + mm] * sc;
                const float z1 = tile[(2 * pl + 1) * COLS + mm] * sc;
                const float c = a.rope[mm * half + p], sn = a.rope[kMaxR * half + mm * half + p];
                const float o0 = z0 * c - z1 * sn, o1 = z1 * c + z0 * sn;
                if (is_q) {
                    a.q[size_t(mm) * a.q_dim + head * h + p] = o0;
                    a.q[size_t(mm) * a.q_dim + head * h + p + half] = o1;
                } else {
                    const int slot = a.ctx_len + mm;
                    const int page = a.block_table[slot >> 4], tk = slot & 15;
                    __bf16* kp = a.kpool + (size_t(page) * a.n_kv_heads + head) * (16 * h);
                    kp[((p >> 3) * 16 + tk) * 8 + (p & 7)] = static_cast<__bf16>(o0);
                    const int p2 = p + half;
                    kp[((p2 >> 3) * 16 + tk) * 8 + (p2 & 7)] = static_cast<__bf16>(o1);
                }
            }
        } else {
            for (int e = tid; e < kGroupRows * r; e += kGemmWaves * 64) {
                const int nl = e % kGroupRows, mm = e / kGroupRows;
                const int rel = row0 + nl - a.q_dim - a.kv_dim;
                if (rel < a.kv_dim) {
                    const int head = rel / h, j = rel % h;
                    const int slot = a.ctx_len + mm;
                    const int page = a.block_table[slot >> 4], tk = slot & 15;
                    __bf16* vp = a.vpool + (size_t(page) * a.n_kv_heads + head) * (16 * h);
                    vp[j * 16 + tk] = static_cast<__bf16>(tile[nl * COLS + mm] * row_scale[mm]);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Embedding gather + per-call set-up: x[m] = E[token m]; partial sums of squares per 64-column
// group; the rotation table cos/sin(pos * theta^(-2j/h)) in fp64; clears the counters.
// ------------------------------------------------------------------------------------------
struct EmbedArgs {
    const __bf16* embed;
    const int32_t* tokens;
    int32_t r, d, vocab;
    float* x;
    float* ss_out;
    float* rope;
    int32_t ctx_len, head_dim;
    float theta;
    int32_t* counters;
    int32_t n_counters;
    int32_t* acounters;
    int32_t n_acounters;
    unsigned long long* best;  // [32] arg-max keys, cleared here
};

__global__ __launch_bounds__(64) void k_embed(EmbedArgs a) {
    const int g = blockIdx.x, lane = threadIdx.x;
    const int n = g * 64 + lane;
    for (int m = 0; m < a.r; ++m) {
        int tok = a.tokens[m];
        tok = tok < 0 ? 0 : (tok >= a.vocab ? a.vocab - 1 : tok);
        float v = 0.f;
        if (n < a.d) {
            v = static_cast<float>(a.embed[size_t(tok) * a.d + n]);
            a.x[size_t(m) * a.d + n] = v;
        }
        float ss = v * v;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) ss += __shfl_xor(ss, o);
        if (lane == 0) a.ss_out[g * kMaxR + m] = ss;
    }
    // rotation table, spread over the workgroups; angles in fp64 so long contexts stay exact
    const int half = a.head_dim >> 1;
    for (int e = n; e < a.r * half; e += gridDim.x * 64) {
        const int m = e / half, j = e % half;
        const double ang = double(a.ctx_len + m) * pow(double(a.theta), -2.0 * j / a.head_dim);
        a.rope[m * half + j] = float(cos(ang));
        a.rope[kMaxR * half + m * half + j] = float(sin(ang));
    }
    for (int e = n; e < a.n_counters; e += gridDim.x * 64) a.counters[e] = 0;
    for (int e = n; e < a.n_acounters; e += gridDim.x * 64) a.acounters[e] = 0;
    if (n < kMaxR) a.best[n] = 0ull;
}

// ------------------------------------------------------------------------------------------
// Chain verification attention (the target never needs tree attention: Cache Correction, last
// paragraph).  Rows = the G query heads sharing one KV head x the r candidates; row (m, g) sees
// keys at positions <= ctx_len + m.  Task = (kv head, pair of 16-row tiles, cut of the page
// list).  Per 16-token page: S^T = K Q^T on the matrix pipe (K page stored in operand order),
// online softmax per row with wavefront-level reductions, O^T += V^T P^T with the probability
// tile fed straight from the accumulator registers.  Wavefront partials (max, sum, O) meet in
// LDS, cuts meet in global partials merged by the last workgroup to arrive.
// ------------------------------------------------------------------------------------------
struct AttnArgs {
    const float* q;  // [r][q_dim]
    const __bf16* kpool;
    const __bf16* vpool;
    const int32_t* block_table;
    int32_t r, G, n_kv_heads, q_dim, ctx_len;
    int32_t n_pages_used;  // ceil((ctx_len + r) / 16)
    int32_t splits, pages_per_split, row_pairs;
    float inv_sqrt_h;
    float* part;      // [task][32*(H+2)] : M[32], L[32], O[32][H]
    int32_t* counters;
    float* att;       // [r][q_dim]
};

template <int H>
__global__ __launch_bounds__(kAttnWaves * 64) void k_attn(AttnArgs a) {
    constexpr int ST = H / 32;  // k-steps of the QK^T contraction
    constexpr int HT = H / 16;  // 16-row tiles of O^T
    constexpr int PART = 32 * (H + 2);
    __shared__ float lds[kAttnWaves * PART];
    __shared__ float wgt[64 * 32];
    __shared__ int is_last;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    int task = blockIdx.x;
    const int split = task % a.splits;
    task /= a.splits;
    const int pair = task % a.row_pairs;
    const int kvh = task / a.row_pairs;
    const int R = a.G * a.r;
    const int col = lane & 15, kq = lane >> 4;

    // Q^T operand: lane holds row rho, head elements 32*st + 8*kq .. +8, as high and low halves
    bf16x8 qh[2][ST], ql[2][ST];
    int mrow[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int rho = (pair * 2 + t) * 16 + col;
        const bool ok = rho < R;
        const int m = ok ? rho / a.G : 0, gl = ok ? rho % a.G : 0;
        mrow[t] = ok ? m : -1;
        const float* qp = a.q + size_t(m) * a.q_dim + (kvh * a.G + gl) * H + kq * 8;
#pragma unroll
        for (int st = 0; st < ST; ++st) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = ok ? qp[st * 32 + e] * a.inv_sqrt_h : 0.f;
                __bf16 hi, lo;
                split_bf16(v, hi, lo);
                qh[t][st][e] = hi;
                ql[t][st][e] = lo;
            }
        }
    }

    floatx4 o[2][HT];
    float mx[2], sum[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        mx[t] = -1e30f;
        sum[t] = 0.f;
#pragma unroll
        for (int i = 0; i < HT; ++i) o[t][i] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    const int pg0 = split * a.pages_per_split;
    const int pg1 = min(a.n_pages_used, pg0 + a.pages_per_split);
    for (int pg = pg0 + wave; pg < pg1; pg += kAttnWaves) {
        const int pid = a.block_table[pg];
        const size_t base = (size_t(pid) * a.n_kv_heads + kvh) * (16 * H);
        const bf16x8* kp = reinterpret_cast<const bf16x8*>(a.kpool + base) + lane;
        bf16x8 kf[ST];
#pragma unroll
        for (int st = 0; st < ST; ++st) kf[st] = kp[st * 64];
        short4v vf[HT];
        const short4v* vp = reinterpret_cast<const short4v*>(a.vpool + base) + (col * 4 + kq);
#pragma unroll
        for (int i = 0; i < HT; ++i) vf[i] = vp[i * 64];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            floatx4 s = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int st = 0; st < ST; ++st) {
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[st], qh[t][st], s, 0, 0, 0);
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[st], ql[t][st], s, 0, 0, 0);
            }
            // lane holds keys kq*4 + v of this page for row `col` of tile t
            const int limit = a.ctx_len + mrow[t];  // last visible position (mrow = -1: nothing real)
            float pmax = -1e30f;
            bool ok[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                ok[v] = mrow[t] >= 0 && (pg * 16 + kq * 4 + v) <= limit;
                if (ok[v]) pmax = fmaxf(pmax, s[v]);
            }
            pmax = fmaxf(pmax, __shfl_xor(pmax, 16));
            pmax = fmaxf(pmax, __shfl_xor(pmax, 32));
            const float mnew = fmaxf(mx[t], pmax);
            const float alpha = expf(mx[t] - mnew);
            float p[4], psum = 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                p[v] = ok[v] ? expf(s[v] - mnew) : 0.f;
                psum += p[v];
            }
            psum += __shfl_xor(psum, 16);
            psum += __shfl_xor(psum, 32);
            sum[t] = sum[t] * alpha + psum;
            mx[t] = mnew;
            short4v ph, pl;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                __bf16 hi, lo;
                split_bf16(p[v], hi, lo);
                ph[v] = __builtin_bit_cast(short, hi);
                pl[v] = __builtin_bit_cast(short, lo);
            }
#pragma unroll
            for (int i = 0; i < HT; ++i) {
                floatx4 acc = o[t][i];
                acc[0] *= alpha; acc[1] *= alpha; acc[2] *= alpha; acc[3] *= alpha;
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vf[i], ph, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vf[i], pl, acc, 0, 0, 0);
                o[t][i] = acc;
            }
        }
    }

    // wavefront partials -> LDS: M[32], L[32], O[32 rows][H]
    float* mine = lds + wave * PART;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        if (kq == 0) {
            mine[t * 16 + col] = mx[t];
            mine[32 + t * 16 + col] = sum[t];
        }
#pragma unroll
        for (int i = 0; i < HT; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) mine[64 + (t * 16 + col) * H + i * 16 + kq * 4 + v] = o[t][i][v];
    }
    __syncthreads();
    // merge the wavefronts (fixed order) into slot 0 of LDS
    if (tid < 32) {
        float mg = -1e30f;
        for (int w = 0; w < kAttnWaves; ++w) mg = fmaxf(mg, lds[w * PART + tid]);
        float l = 0.f;
        for (int w = 0; w < kAttnWaves; ++w) {
            const float f = expf(lds[w * PART + tid] - mg);
            wgt[w * 32 + tid] = f;
            l += f * lds[w * PART + 32 + tid];
        }
        wgt[kAttnWaves * 32 + tid] = mg;
        wgt[(kAttnWaves + 1) * 32 + tid] = l;
    }
    __syncthreads();
    float* gpart = a.part + size_t(blockIdx.x) * PART;
    for (int e = tid; e < 32 * H; e += kAttnWaves * 64) {
        const int row = e / H;
        float acc = 0.f;
        for (int w = 0; w < kAttnWaves; ++w) acc += wgt[w * 32 + row] * lds[w * PART + 64 + e];
        st_agent(gpart + 64 + e, acc);
    }
    if (tid < 32) {
        st_agent(gpart + tid, wgt[kAttnWaves * 32 + tid]);
        st_agent(gpart + 32 + tid, wgt[(kAttnWaves + 1) * 32 + tid]);
    }
    wait_stores();
    __syncthreads();
    const int cidx = kvh * a.row_pairs + pair;
    if (tid == 0) {
        const int prev = __hip_atomic_fetch_add(&a.counters[cidx], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        is_last = (prev == a.splits - 1);
    }
    __syncthreads();
    if (!is_last) return;
    const float* base = a.part + size_t(blockIdx.x - split) * PART;
    // merge the cuts in cut order: one thread per (row, cut) fetches max and sum, then per row
    for (int e = tid; e < 32 * a.splits; e += kAttnWaves * 64) {
        const int row = e & 31, sp = e >> 5;
        lds[e] = ld_agent(base + size_t(sp) * PART + row);
        lds[2048 + e] = ld_agent(base + size_t(sp) * PART + 32 + row);
    }
    __syncthreads();
    if (tid < 32) {
        float mg = -1e30f;
        for (int sp = 0; sp < a.splits; ++sp) mg = fmaxf(mg, lds[sp * 32 + tid]);
        float l = 0.f;
        for (int sp = 0; sp < a.splits; ++sp) {
            const float f = expf(lds[sp * 32 + tid] - mg);
            wgt[sp * 32 + tid] = f;
            l += f * lds[2048 + sp * 32 + tid];
        }
        lds[4096 + tid] = l;
    }
    __syncthreads();
    for (int e = tid; e < 32 * H; e += kAttnWaves * 64) {
        const int row = e / H, hh = e % H;
        const int rho = pair * 32 + row;
        if (rho >= R) continue;
        float acc = 0.f;
        int sp = 0;
        for (; sp + 4 <= a.splits; sp += 4) {
            const float v0 = ld_agent(base + size_t(sp) * PART + 64 + e);
            const float v1 = ld_agent(base + size_t(sp + 1) * PART + 64 + e);
            const float v2 = ld_agent(base + size_t(sp + 2) * PART + 64 + e);
            const float v3 = ld_agent(base + size_t(sp + 3) * PART + 64 + e);
            acc += wgt[sp * 32 + row] * v0;
            acc += wgt[(sp + 1) * 32 + row] * v1;
            acc += wgt[(sp + 2) * 32 + row] * v2;
            acc += wgt[(sp + 3) * 32 + row] * v3;
        }
        for (; sp < a.splits; ++sp) acc += wgt[sp * 32 + row] * ld_agent(base + size_t(sp) * PART + 64 + e);
        const int m = rho / a.G, gl = rho % a.G;
        a.att[size_t(m) * a.q_dim + (kvh * a.G + gl) * H + hh] = acc / lds[4096 + row];
    }
    if (tid == 0) __hip_atomic_store(&a.counters[cidx], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ------------------------------------------------------------------------------------------
// Arg-max over the per-group partials, then greedy prefix acceptance and the correction token
// (overview figure: accept the matching prefix, emit the target's own next token).
// ------------------------------------------------------------------------------------------
struct AcceptArgs {
    const unsigned long long* best;  // [32] packed (logit key, ~index) per row
    int32_t r;
    const int32_t* cand;
    int32_t pending, ctx_len;
    card_verify_result* out;
    int32_t* row_argmax;  // optional
};

__global__ __launch_bounds__(64) void k_accept(AcceptArgs a) {
    __shared__ int pred[kMaxR + 1];
    const int tid = threadIdx.x;
    if (tid < a.r) pred[tid + 1] = int(0xffffffffu - uint32_t(a.best[tid] & 0xffffffffull));
    __syncthreads();
    if (tid == 0) {
        pred[0] = a.pending < 0 ? a.cand[0] : a.pending;
        int j = 0;
        while (j < a.r && a.cand[j] == pred[j]) ++j;
        a.out->accepted_len = j;
        a.out->correction_token = pred[j];
        a.out->kv_first_slot = a.ctx_len;
        a.out->kv_count = j;
    }
    if (a.row_argmax && tid < a.r) a.row_argmax[tid] = pred[tid + 1];
}

// ------------------------------------------------------------------------------------------
// Weight re-layout: canonical row-major bf16 -> tile order.  One thread per 8-element chunk.
// ------------------------------------------------------------------------------------------
enum RowMap { MAP_IDENT = 0, MAP_ROPE = 1, MAP_GATE = 2, MAP_UP = 3 };

struct PackArgs {
    const __bf16* src;  // [src_rows][K]
    __bf16* dst;        // packed matrix base
    int32_t src_rows, K, Ks, n_rows;  // n_rows: packed rows this call fills (incl. zero padding)
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
    reinterpret_cast<bf16x8*>(a.dst)[(size_t(t) * a.Ks + s) * 64 + lane] = v;
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
    a.v_out[id] = static_cast<float>(a.vpool[base + j * 16 + tk]);
}

}  // namespace card
