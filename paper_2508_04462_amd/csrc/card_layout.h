// Host-side description of where everything lives: the packed weight blob, the workspace,
// of the persistent verify kernel.  Plain structs, passed to kernels by value.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "card.h"

namespace card {

constexpr int kTileN = 16;     // rows of one matrix-instruction tile (output features)
constexpr int kTileK = 32;     // contraction depth of one bf16 16x16x32 matrix instruction
constexpr int kMaxR = 32;
constexpr int kKvBlock = 16;
// tiles a workgroup accumulates side by side (batch width) per kind of matrix
constexpr int kNbQkv = 2, kNbOne = 1, kNbWide = 8;
constexpr int kFlagCopies = 32;  // copies of the barrier flags (256 words each): pollers spread over them
constexpr uint32_t kStampMagic = 0x43415244u;  // "CARD"
constexpr uint32_t kWsMagic = 0x57534b31u;     // workspace control words initialised ("WSK1"), word kBarMagic
// words of the barrier block: [1] exit counter, [2] error flag, [3] barrier epoch, [4] magic
constexpr int kBarExit = 1, kBarError = 2, kBarEpoch = 3, kBarMagic = 4;

#ifdef __HIPCC__
#define CARD_HD __host__ __device__
#else
#define CARD_HD
#endif

constexpr int kStreamWaves = 4;  // wavefront pairs of a workgroup: they cut the contraction four ways

// One matrix as Nt n-tiles x Ks k-steps of 1 KiB fragments [64 lanes][8 bf16]: lane l of
// fragment (t, s) holds row 16t + l%16, columns 32s + 8*(l/16) .. +8; rows / columns beyond
// N / K are zero.  Fragments are stored in STREAM ORDER, the order in which the verify kernel
// consumes them on a grid of nwg workgroups: tile t belongs to position p = t % nwg of the grid
// (its j-th tile, j = t / nwg), k-step s to the wavefront pair w with w*Ks/4 <= s < (w+1)*Ks/4.
// Memory holds position after position, inside a position pair after pair, and inside a pair
// the tiles NB at a time ("batch"): batch, then k-step, then tile of the batch.  Every wavefront
// pair therefore reads ONE contiguous run per matrix.
struct MatDesc {
    size_t off;  // byte offset inside the packed blob (layer matrices: relative to the layer base)
    int32_t N, K, Nt, Ks, NB;
    size_t bytes() const { return size_t(Nt) * Ks * 1024; }
};

// Tiles of grid position p, the k-steps [s0, s1) of pair w, and the index of the pair's first
// fragment in the matrix.
struct StreamRun {
    int32_t cnt, s0, s1;
    int64_t first;
};
CARD_HD inline StreamRun stream_run(int32_t Nt, int32_t Ks, int32_t nwg, int32_t p, int32_t w) {
    StreamRun r;
    const int32_t full = Nt / nwg, rem = Nt % nwg;
    r.cnt = full + (p < rem ? 1 : 0);
    r.s0 = (w * Ks) / kStreamWaves;
    r.s1 = ((w + 1) * Ks) / kStreamWaves;
    r.first = (int64_t(full) * p + (p < rem ? p : rem)) * Ks + int64_t(r.cnt) * r.s0;
    return r;
}
// Index of fragment (tile t, k-step s) in stream order.
CARD_HD inline int64_t stream_frag_index(int32_t Nt, int32_t Ks, int32_t NB, int32_t nwg, int32_t t, int32_t s) {
    const int32_t p = t % nwg, j = t / nwg;
    int32_t w = 0;
    while (w + 1 < kStreamWaves && s >= ((w + 1) * Ks) / kStreamWaves) ++w;
    const StreamRun r = stream_run(Nt, Ks, nwg, p, w);
    const int32_t b = j / NB, i = j % NB;
    const int32_t nv = r.cnt - b * NB < NB ? r.cnt - b * NB : NB;
    return r.first + int64_t(b) * NB * (r.s1 - r.s0) + int64_t(s - r.s0) * nv + i;
}

struct Layout {
    bool ok;
    // packed weights
    size_t embed_off, lm_off, g_final_off, stamp_off, layer0_off, layer_stride, weight_bytes;
    MatDesc qkv, wo, gu, wd, lm;  // layer matrices relative to the layer base; lm absolute
    size_t g_attn_off, g_ffn_off; // relative to the layer base
    size_t ws_bytes;
    // workspace of the persistent kernel (byte offsets) and strides in elements
    size_t m_xres_off, m_xfrag_off, m_ss_off, m_qfrag_off, m_attfrag_off, m_actfrag_off, m_apart_off, m_bar_off,
        m_acount_off, m_flags_off, m_best_off, m_rope_off, m_topk_off, m_lse_off, m_out_off, m_dpart_off,
        m_dcount_off;
    size_t xfrag_stride, attfrag_stride, actfrag_stride, qfrag_stride;
    int32_t m_attn_max_splits;
};

inline int32_t ceil_div(int64_t a, int64_t b) { return int32_t((a + b - 1) / b); }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline MatDesc make_mat(size_t off, int32_t N, int32_t K, int32_t NB) {
    MatDesc m;
    m.off = off;
    m.N = N;
    m.K = K;
    m.NB = NB;
    m.Nt = ceil_div(N, kTileN);
    m.Ks = ceil_div(K, kTileK);
    return m;
}

inline bool cfg_valid(const card_model_cfg* c) {
    if (!c) return false;
    if (c->n_layers <= 0 || c->d_model <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->d_ffn <= 0 ||
        c->vocab <= 1)
        return false;
    if (c->head_dim != 64 && c->head_dim != 128) return false;
    if (c->d_model % 64 || c->d_ffn % 8) return false;
    if (c->n_q_heads % c->n_kv_heads) return false;
    if (c->kv_block != kKvBlock) return false;
    if (c->max_ctx <= 0 || c->max_ctx % kKvBlock) return false;
    if (c->max_r < 1 || c->max_r > kMaxR) return false;
    if (!(c->rope_theta > 0.f) || !(c->rms_eps >= 0.f)) return false;
    if (c->grid_wgs < 0 || c->grid_wgs > 256) return false;
    return true;
}

inline Layout make_layout(const card_model_cfg* c) {
    Layout L = {};
    if (!cfg_valid(c)) return L;
    const int32_t d = c->d_model, h = c->head_dim, qd = c->n_q_heads * h, kvd = c->n_kv_heads * h;
    size_t off = 0;
    L.embed_off = off;
    off = align_up(off + size_t(c->vocab) * d * 2, 1024);
    L.lm = make_mat(off, c->vocab, d, kNbWide);
    L.lm_off = off;
    off = align_up(off + L.lm.bytes(), 1024);
    L.g_final_off = off;
    off = align_up(off + size_t(d) * 4, 1024);
    L.stamp_off = off;  // {magic, grid size the stream order was laid out for}
    off += 1024;
    L.layer0_off = off;
    size_t lo = 0;
    L.qkv = make_mat(lo, qd + 2 * kvd, d, kNbQkv);
    lo += L.qkv.bytes();
    L.wo = make_mat(lo, d, qd, kNbOne);
    lo += L.wo.bytes();
    L.gu = make_mat(lo, 2 * c->d_ffn, d, kNbWide);
    lo += L.gu.bytes();
    L.wd = make_mat(lo, d, c->d_ffn, kNbOne);
    lo += L.wd.bytes();
    L.g_attn_off = lo;
    lo = align_up(lo + size_t(d) * 4, 1024);
    L.g_ffn_off = lo;
    lo = align_up(lo + size_t(d) * 4, 1024);
    L.layer_stride = lo;
    L.weight_bytes = L.layer0_off + size_t(c->n_layers) * L.layer_stride;
    // the kernel addresses a matrix with 32-bit byte offsets
    constexpr size_t k4G = size_t(1) << 32;
    if (L.qkv.bytes() >= k4G || L.wo.bytes() >= k4G || L.gu.bytes() >= k4G || L.wd.bytes() >= k4G || L.lm.bytes() >= k4G)
        return L;

    // workspace
    size_t w = 0;
    auto take = [&](size_t bytes) {
        size_t at = w;
        w = align_up(w + bytes, 256);
        return at;
    };
    const int32_t G = c->n_q_heads / c->n_kv_heads;
    // persistent kernel: one copy of every hand-over buffer per layer and phase
    auto frag_elems = [](int32_t K) { return size_t(ceil_div(K, kTileK)) * 4 * kMaxR * 16; };
    const int32_t versions = 2 * c->n_layers + 1;
    L.xfrag_stride = frag_elems(d);
    L.attfrag_stride = frag_elems(qd);
    L.actfrag_stride = frag_elems(c->d_ffn);
    L.qfrag_stride = size_t(c->n_q_heads) * kMaxR * h * 2;
    L.m_xres_off = take(size_t(versions) * kMaxR * d * 4);
    L.m_xfrag_off = take(size_t(versions) * L.xfrag_stride * 2);
    L.m_ss_off = take(size_t(versions) * (d / 16) * kMaxR * 4);
    L.m_qfrag_off = take(size_t(c->n_layers) * L.qfrag_stride * 2);
    L.m_attfrag_off = take(size_t(c->n_layers) * L.attfrag_stride * 2);
    L.m_actfrag_off = take(size_t(c->n_layers) * L.actfrag_stride * 2);
    L.m_attn_max_splits = 32;
    L.m_apart_off = take(size_t(c->n_kv_heads) * (2 * G) * L.m_attn_max_splits * 16 * (h + 2) * 4);
    L.m_bar_off = take(256);
    L.m_flags_off = take(size_t(kFlagCopies) * 1024);
    L.m_acount_off = take(size_t(c->n_kv_heads) * (2 * G) * 4);
    L.m_best_off = take(size_t(kMaxR) * 8);
    L.m_rope_off = take(size_t(kMaxR) * h * 4);
    L.m_topk_off = take(size_t(256) * kMaxR * 16 * 8);  // per workgroup and row: sixteen best keys
    L.m_lse_off = take(size_t(256) * kMaxR * 2 * 4);    // per workgroup and row: (max, sum of exp)
    L.m_out_off = take(64);                             // where a draft-side call parks the verify result
    // down-projection at r > 8: the four workgroups of a group each hold a quarter of K of the
    // group's tiles; per tile four partial blocks of 16 x 32 fp32, and one arrival counter per
    // four tiles
    L.m_dpart_off = take(size_t(L.wd.Nt) * kStreamWaves * 16 * kMaxR * 4);
    L.m_dcount_off = take(size_t(ceil_div(L.wd.Nt, 4)) * 4);
    L.ws_bytes = w;
    L.ok = true;
    return L;
}

}  // namespace card
