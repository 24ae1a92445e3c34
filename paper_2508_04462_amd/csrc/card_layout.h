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

// One matrix in tile order: [Nt n-tiles][Ks k-steps][64 lanes][8 bf16]; lane l of tile (t, s)
// holds row 16t + l%16, columns 32s + 8*(l/16) .. +8.  Rows / columns beyond N / K are zero.
struct MatDesc {
    size_t off;  // byte offset inside the packed blob (layer matrices: relative to the layer base)
    int32_t N, K, Nt, Ks;
    size_t bytes() const { return size_t(Nt) * Ks * 1024; }
};

struct Layout {
    bool ok;
    // packed weights
    size_t embed_off, lm_off, g_final_off, layer0_off, layer_stride, weight_bytes;
    MatDesc qkv, wo, gu, wd, lm;  // layer matrices relative to the layer base; lm absolute
    size_t g_attn_off, g_ffn_off; // relative to the layer base
    size_t ws_bytes;
    // workspace of the persistent kernel (byte offsets) and strides in elements
    size_t m_xres_off, m_xfrag_off, m_ss_off, m_qfrag_off, m_attfrag_off, m_actfrag_off, m_apart_off, m_bar_off,
        m_acount_off, m_flags_off, m_best_off, m_rope_off;
    size_t xfrag_stride, attfrag_stride, actfrag_stride, qfrag_stride;
    int32_t m_attn_max_splits;
};

inline int32_t ceil_div(int64_t a, int64_t b) { return int32_t((a + b - 1) / b); }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline MatDesc make_mat(size_t off, int32_t N, int32_t K) {
    MatDesc m;
    m.off = off;
    m.N = N;
    m.K = K;
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
    return true;
}

inline Layout make_layout(const card_model_cfg* c) {
    Layout L = {};
    if (!cfg_valid(c)) return L;
    const int32_t d = c->d_model, h = c->head_dim, qd = c->n_q_heads * h, kvd = c->n_kv_heads * h;
    size_t off = 0;
    L.embed_off = off;
    off = align_up(off + size_t(c->vocab) * d * 2, 1024);
    L.lm = make_mat(off, c->vocab, d);
    L.lm_off = off;
    off = align_up(off + L.lm.bytes(), 1024);
    L.g_final_off = off;
    off = align_up(off + size_t(d) * 4, 1024);
    L.layer0_off = off;
    size_t lo = 0;
    L.qkv = make_mat(lo, qd + 2 * kvd, d);
    lo += L.qkv.bytes();
    L.wo = make_mat(lo, d, qd);
    lo += L.wo.bytes();
    L.gu = make_mat(lo, 2 * c->d_ffn, d);
    lo += L.gu.bytes();
    L.wd = make_mat(lo, d, c->d_ffn);
    lo += L.wd.bytes();
    L.g_attn_off = lo;
    lo = align_up(lo + size_t(d) * 4, 1024);
    L.g_ffn_off = lo;
    lo = align_up(lo + size_t(d) * 4, 1024);
    L.layer_stride = lo;
    L.weight_bytes = L.layer0_off + size_t(c->n_layers) * L.layer_stride;

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
    L.m_flags_off = take(4 * 1024);
    L.m_acount_off = take(size_t(c->n_kv_heads) * (2 * G) * 4);
    L.m_best_off = take(size_t(kMaxR) * 8);
    L.m_rope_off = take(size_t(kMaxR) * h * 4);
    L.ws_bytes = w;
    L.ok = true;
    return L;
}

}  // namespace card
