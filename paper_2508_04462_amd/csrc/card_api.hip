// C ABI of libcard: argument checks and the launch sequence of one verification step.
#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <hip/hip_runtime.h>

#include <vector>

#include "card.h"

#ifndef CARD_STATIC_SCRATCH_BYTES
#define CARD_STATIC_SCRATCH_BYTES (32u << 20)
#endif
#include "card_pack.hip"
#include "card_verify.hip"

using namespace card;

namespace {

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

inline int launch_status() { return hipGetLastError() == hipSuccess ? CARD_OK : CARD_EDEVICE; }

unsigned long long* g_ts_buf = nullptr;
int g_ts_layer = 0;

// Benchmark hook: event pairs around the verify kernel.  One user at a time (the lock only keeps
// enable / disable / collect and a concurrent card_verify from tearing the vectors).  The events
// are destroyed by card_profile_disable, never by a static destructor: at process exit the HIP
// runtime may already be gone.
struct Profile {
    std::mutex mu;
    std::atomic<bool> on{false};
    int used = 0;
    std::vector<hipEvent_t> start, stop;
};
Profile& prof() {
    static Profile* p = new Profile;  // leaked on purpose: no destructor runs after HIP teardown
    return *p;
}

struct ProfScope {
    hipStream_t st;
    hipEvent_t stop = nullptr;
    explicit ProfScope(hipStream_t s) : st(s) {
        Profile& p = prof();
        if (!p.on) return;
        std::lock_guard<std::mutex> g(p.mu);
        if (p.on && p.used < int(p.start.size())) {
            const int idx = p.used++;
            (void)hipEventRecord(p.start[idx], st);
            stop = p.stop[idx];
        }
    }
    ~ProfScope() {
        if (stop) (void)hipEventRecord(stop, st);
    }
};

constexpr int kMaxDevices = 64;

// Compute units of the current device (cached per device id).
int cu_count() {
    static std::atomic<int> cus[kMaxDevices];
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    n = cus[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Workgroups of the verify kernel: cfg->grid_wgs if the caller fixed it, else one per compute
// unit; at most 256 (the barrier polls 256 flags), never more than the compute units there are
// (every workgroup needs a compute unit of its own: the grid meets at barriers).
int grid_size(const card_model_cfg* cfg) {
    const int cus = cu_count();
    int n = cus > 256 ? 256 : cus;
    if (cfg && cfg->grid_wgs > 0) {
        if (cfg->grid_wgs > n) return 0;
        n = cfg->grid_wgs;
    }
    return n;
}

// The kernel synchronises its workgroups through flags in memory, so all of them have to be
// resident at once.  It is launched as an ordinary kernel: one workgroup fills a compute unit
// (158.5 KiB of its LDS, 512 threads with 256 registers each), the grid is no larger than the
// number of compute units, and the occupancy query below confirms that the device can hold a
// workgroup per compute unit, so on an otherwise idle device the dispatcher places all of them.
// Should other work hold compute units for longer than the kernel's bounded waits, the step ends
// with accepted_len = -1 instead of hanging.
template <int MT, int H, bool PK, bool DR>
int launch_mega(MegaArgs& a, hipStream_t st) {
    static std::atomic<int> fits[kMaxDevices];  // 0 unknown, 1 yes, -1 no
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CARD_EDEVICE;
    int f = fits[dev].load(std::memory_order_relaxed);
    if (f == 0) {
        int per_cu = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_verify<MT, H, PK, DR>, kBlockThreads, 0) != hipSuccess)
            return CARD_EDEVICE;
        f = per_cu >= 1 ? 1 : -1;
        fits[dev].store(f, std::memory_order_relaxed);
    }
    if (f < 0 || a.nwg > cu_count()) return CARD_EDEVICE;
    hipLaunchKernelGGL((k_verify<MT, H, PK, DR>), dim3(a.nwg), dim3(kBlockThreads), 0, st, a);
    return launch_status();
}

// Scratch of the entry point that allocates nothing: what card_verify takes as `workspace_dev`,
// at a fixed place in the code object.  In host code the name is a stand-in, not a device address:
// the address of this device's copy comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticWsBytes = size_t(CARD_STATIC_SCRATCH_BYTES);
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];

struct StaticWs {
    void* ptr = nullptr;       // device address of `scratch` on this device
    bool prepared = false;     // k_ws_init has been enqueued for `cfg`'s layout
    card_model_cfg cfg = {};
};
StaticWs g_static[kMaxDevices];
std::mutex g_static_mu;

// Draft-side options of a step (card_draft_level): tree rows and the per-row top-k.
struct TreeOpt {
    const int32_t* row_pos;
    int32_t first_slot;
    const uint32_t* mask;
    int32_t mask_words, mask_base;
    int32_t topk;
    int32_t* topk_tok;
    float* topk_prob;
};

// One persistent kernel runs the whole step (card_verify.hip).
int verify_impl(const card_model_cfg* cfg, const void* packed, const card_kv* kv, int32_t ctx_len,
                const int32_t* cand, int32_t r, void* workspace, void* stream, card_verify_result* out,
                int32_t* row_argmax, float* logits, const card_sampling* sampling = nullptr,
                const TreeOpt* tree = nullptr) {
    if (!cfg || !packed || !kv || !cand || !workspace || (!out && !tree)) return CARD_EINVAL;
    const Layout L = make_layout(cfg);
    if (!L.ok) return CARD_EINVAL;
    if (!kv->k_pages || !kv->v_pages || !kv->block_table || kv->n_pages <= 0) return CARD_EINVAL;
    // one layer of a page pool is addressed with 32-bit byte offsets
    if (size_t(kv->n_pages) * cfg->n_kv_heads * 16 * cfg->head_dim * 2 >= (size_t(1) << 32)) return CARD_EINVAL;
    if (r < 1 || r > cfg->max_r) return CARD_ERANGE;
    if (ctx_len < 0) return CARD_EINVAL;
    const int32_t slot0 = tree ? tree->first_slot : ctx_len;
    if (int64_t(slot0) + r > cfg->max_ctx) return CARD_ECAPACITY;
    if (tree) {
        if (!tree->row_pos || !tree->mask || !tree->topk_tok || !tree->topk_prob) return CARD_EINVAL;
        if (tree->mask_words < 1 || tree->mask_words > 32 || tree->topk < 1 || tree->topk > 16) return CARD_ERANGE;
        if (tree->mask_base < 0 || tree->mask_base % kKvBlock || tree->mask_base > ctx_len) return CARD_EINVAL;
        if (slot0 < ctx_len || int64_t(slot0) + r > int64_t(tree->mask_base) + 32 * tree->mask_words) return CARD_ERANGE;
    }
    const int cus = grid_size(cfg);
    if (cus <= 0) return CARD_EDEVICE;

    char* ws = static_cast<char*>(workspace);
    const int h = cfg->head_dim;
    MegaArgs a = {};
    a.L = cfg->n_layers;
    a.d = cfg->d_model;
    a.qd = cfg->n_q_heads * h;
    a.kvd = cfg->n_kv_heads * h;
    a.h = h;
    a.Hkv = cfg->n_kv_heads;
    a.G = cfg->n_q_heads / cfg->n_kv_heads;
    a.F = cfg->d_ffn;
    a.V = cfg->vocab;
    a.r = r;
    a.rp = (r + 7) / 8 * 8;
    a.ctx_len = ctx_len;
    a.nwg = cus;
    a.eps = cfg->rms_eps;
    a.inv_d = 1.0f / float(cfg->d_model);
    a.theta = cfg->rope_theta;
    a.inv_sqrt_h = 1.4426950408889634f / sqrtf(float(h));  // log2(e)/sqrt(h): the softmax runs on exp2
    a.wbase = static_cast<const char*>(packed);
    a.embed_off = L.embed_off;
    a.g_final_off = L.g_final_off;
    a.layer0_off = L.layer0_off;
    a.stamp = reinterpret_cast<const uint32_t*>(a.wbase + L.stamp_off);
    a.layer_stride = L.layer_stride;
    a.g_attn_off = L.g_attn_off;
    a.g_ffn_off = L.g_ffn_off;
    a.qkv = L.qkv;
    a.wo = L.wo;
    a.gu = L.gu;
    a.wd = L.wd;
    a.lm = L.lm;
    a.kpool = static_cast<__bf16*>(kv->k_pages);
    a.vpool = static_cast<__bf16*>(kv->v_pages);
    a.pool_layer_elems = size_t(kv->n_pages) * cfg->n_kv_heads * 16 * h;
    a.block_table = kv->block_table;
    a.pages_used = ceil_div(slot0 + r, kKvBlock);
    a.slot0 = slot0;
    a.old_end = tree ? tree->mask_base : ctx_len;
    a.row_tiles = ceil_div(a.G * r, 16);
    // Cut the context so that a workgroup's share fits the page buffers of its wavefronts (all of
    // its old-context pages are then in flight before the barrier in front of attention), as long
    // as every task still gets a workgroup of its own; beyond that the shares grow instead.
    // The cut length is a function of the context length in steps of 512 tokens, the grid and
    // the kernel (r <= 8, <= 16, <= 32), not of r itself: a row's keys are then cut, summed and
    // merged in the same order whether a step of eight rows or a plain decode step computes it,
    // and verification reproduces the plain decode's logits bit for bit (same kernel, same
    // 512-token stretch).
    const int share = kMegaWaves * (h == 128 ? 2 : 4);
    const int r_kernel = r <= 8 ? 8 : (r <= 16 ? 16 : 32);
    const int max_cuts = std::min<int>(L.m_attn_max_splits, std::max(1, cus / (a.Hkv * ceil_div(a.G * r_kernel, 16))));
    const int pages_stretch = ceil_div(a.pages_used, 32) * 32;
    a.pages_per_split = std::max(share, ceil_div(pages_stretch, max_cuts));
    a.a_splits = ceil_div(a.pages_used, a.pages_per_split);
    a.xres = reinterpret_cast<float*>(ws + L.m_xres_off);
    a.xfrag = reinterpret_cast<__bf16*>(ws + L.m_xfrag_off);
    a.ss = reinterpret_cast<float*>(ws + L.m_ss_off);
    a.qfrag = reinterpret_cast<__bf16*>(ws + L.m_qfrag_off);
    a.attfrag = reinterpret_cast<__bf16*>(ws + L.m_attfrag_off);
    a.actfrag = reinterpret_cast<__bf16*>(ws + L.m_actfrag_off);
    a.apart = reinterpret_cast<float*>(ws + L.m_apart_off);
    a.xfrag_stride = L.xfrag_stride;
    a.attfrag_stride = L.attfrag_stride;
    a.actfrag_stride = L.actfrag_stride;
    a.qfrag_stride = L.qfrag_stride;
    a.rope = reinterpret_cast<float*>(ws + L.m_rope_off);
    a.best = reinterpret_cast<unsigned long long*>(ws + L.m_best_off);
    a.bar = reinterpret_cast<uint32_t*>(ws + L.m_bar_off);
    a.acount = reinterpret_cast<uint32_t*>(ws + L.m_acount_off);
    a.dpart = reinterpret_cast<float*>(ws + L.m_dpart_off);
    a.dcount = reinterpret_cast<uint32_t*>(ws + L.m_dcount_off);
    a.flags = reinterpret_cast<uint32_t*>(ws + L.m_flags_off);
    a.cand = cand;
    if (tree) {
        a.row_pos = tree->row_pos;
        a.tmask = tree->mask;
        a.tmask_words = tree->mask_words;
        a.tmask_base = tree->mask_base;
        a.topk = tree->topk;
        a.topk_tok = tree->topk_tok;
        a.topk_prob = tree->topk_prob;
        a.topk_part = reinterpret_cast<unsigned long long*>(ws + L.m_topk_off);
        a.lse_part = reinterpret_cast<float*>(ws + L.m_lse_off);
        if (!out) out = reinterpret_cast<card_verify_result*>(ws + L.m_out_off);
    }
    a.pending = kv->pending_token;
    if (sampling && sampling->temperature > 0.f) {
        a.inv_temp = 1.0f / sampling->temperature;
        a.seed_lo = uint32_t(sampling->seed & 0xffffffffull);
        a.seed_hi = uint32_t(sampling->seed >> 32);
    }
    a.out = out;
    a.row_argmax = row_argmax;
    a.logits = logits;
    a.ts = g_ts_buf;
    a.ts_layer = g_ts_layer;
    hipStream_t st = as_stream(stream);
    ProfScope ps(st);
    if (tree) {
        if (r <= 8) return h == 128 ? launch_mega<1, 128, true, true>(a, st) : launch_mega<1, 64, true, true>(a, st);
        if (r <= 16) return h == 128 ? launch_mega<1, 128, false, true>(a, st) : launch_mega<1, 64, false, true>(a, st);
        return h == 128 ? launch_mega<2, 128, false, true>(a, st) : launch_mega<2, 64, false, true>(a, st);
    }
    if (r <= 8) return h == 128 ? launch_mega<1, 128, true, false>(a, st) : launch_mega<1, 64, true, false>(a, st);
    if (r <= 16) return h == 128 ? launch_mega<1, 128, false, false>(a, st) : launch_mega<1, 64, false, false>(a, st);
    return h == 128 ? launch_mega<2, 128, false, false>(a, st) : launch_mega<2, 64, false, false>(a, st);
}

}  // namespace

extern "C" {

const char* card_strerror(int status) {
    switch (status) {
        case CARD_OK: return "ok";
        case CARD_EINVAL: return "invalid argument";
        case CARD_ERANGE: return "value out of range";
        case CARD_ECAPACITY: return "KV cache capacity exceeded";
        case CARD_EDEVICE: return "device error";
        case CARD_ESTALE: return "stale cache epoch";
        case CARD_ETOOBIG: return "workspace of this model exceeds the static scratch buffer";
        default: return "unknown status";
    }
}

size_t card_packed_weight_bytes(const card_model_cfg* cfg) {
    const Layout L = make_layout(cfg);
    return L.ok ? L.weight_bytes : 0;
}

size_t card_workspace_bytes(const card_model_cfg* cfg) {
    const Layout L = make_layout(cfg);
    return L.ok ? L.ws_bytes : 0;
}

size_t card_kv_pool_bytes(const card_model_cfg* cfg, int32_t n_pages) {
    if (!cfg_valid(cfg) || n_pages <= 0) return 0;
    return size_t(cfg->n_layers) * n_pages * cfg->n_kv_heads * 16 * cfg->head_dim * 2;
}

int64_t card_stream_frag_index(int32_t n_tiles, int32_t k_steps, int32_t batch, int32_t grid, int32_t t, int32_t s) {
    if (n_tiles <= 0 || k_steps <= 0 || batch <= 0 || grid <= 0 || t < 0 || t >= n_tiles || s < 0 || s >= k_steps)
        return -1;
    return stream_frag_index(n_tiles, k_steps, batch, grid, t, s);
}

int card_weights_pack_tensor(const card_model_cfg* cfg, int32_t tensor, int32_t layer, const void* src_dev,
                             void* packed_dev, void* stream) {
    if (!src_dev || !packed_dev) return CARD_EINVAL;
    const Layout L = make_layout(cfg);
    if (!L.ok) return CARD_EINVAL;
    if (tensor < CARD_T_EMBED || tensor > CARD_T_G_FINAL) return CARD_EINVAL;
    const bool per_layer = !(tensor == CARD_T_EMBED || tensor == CARD_T_LM_HEAD || tensor == CARD_T_G_FINAL);
    if (per_layer && (layer < 0 || layer >= cfg->n_layers)) return CARD_ERANGE;
    hipStream_t st = as_stream(stream);
    char* pb = static_cast<char*>(packed_dev);
    char* lb = pb + L.layer0_off + size_t(per_layer ? layer : 0) * L.layer_stride;
    const int d = cfg->d_model, h = cfg->head_dim, qd = cfg->n_q_heads * h, kvd = cfg->n_kv_heads * h;

    auto copy = [&](char* dst, size_t bytes) {
        return hipMemcpyAsync(dst, src_dev, bytes, hipMemcpyDeviceToDevice, st) == hipSuccess ? CARD_OK
                                                                                               : CARD_EDEVICE;
    };
    auto pack = [&](char* dst, const MatDesc& m, int src_rows, int n_rows, int prow0, int map) {
        PackArgs a = {};
        a.src = static_cast<const __bf16*>(src_dev);
        a.dst = reinterpret_cast<__bf16*>(dst + m.off);
        a.src_rows = src_rows;
        a.K = m.K;
        a.Ks = m.Ks;
        a.n_rows = n_rows;
        a.prow0 = prow0;
        a.map = map;
        a.head_dim = h;
        a.Nt = m.Nt;
        a.NB = m.NB;
        a.nwg = grid_size(cfg);
        if (a.nwg <= 0) return int(CARD_EDEVICE);
        // whoever verifies with these weights must run the grid they were laid out for
        if (hipMemsetD32Async(reinterpret_cast<hipDeviceptr_t>(pb + L.stamp_off), int(kStampMagic), 1, st) != hipSuccess ||
            hipMemsetD32Async(reinterpret_cast<hipDeviceptr_t>(pb + L.stamp_off + 4), a.nwg, 1, st) != hipSuccess)
            return int(CARD_EDEVICE);
        const int64_t total = int64_t(n_rows) * m.Ks * 4;
        hipLaunchKernelGGL(k_pack, dim3(uint32_t((total + 255) / 256)), dim3(256), 0, st, a);
        return launch_status();
    };
    switch (tensor) {
        case CARD_T_EMBED: return copy(pb + L.embed_off, size_t(cfg->vocab) * d * 2);
        case CARD_T_G_FINAL: return copy(pb + L.g_final_off, size_t(d) * 4);
        case CARD_T_G_ATTN: return copy(lb + L.g_attn_off, size_t(d) * 4);
        case CARD_T_G_FFN: return copy(lb + L.g_ffn_off, size_t(d) * 4);
        case CARD_T_WQ: return pack(lb, L.qkv, qd, qd, 0, MAP_ROPE);
        case CARD_T_WK: return pack(lb, L.qkv, kvd, kvd, qd, MAP_ROPE);
        case CARD_T_WV: return pack(lb, L.qkv, kvd, kvd, qd + kvd, MAP_IDENT);
        case CARD_T_WO: return pack(lb, L.wo, d, L.wo.Nt * 16, 0, MAP_IDENT);
        case CARD_T_WG: return pack(lb, L.gu, cfg->d_ffn, cfg->d_ffn, 0, MAP_GATE);
        case CARD_T_WU: return pack(lb, L.gu, cfg->d_ffn, cfg->d_ffn, 0, MAP_UP);
        case CARD_T_WD: return pack(lb, L.wd, d, L.wd.Nt * 16, 0, MAP_IDENT);
        default: {
            MatDesc m = L.lm;
            m.off = 0;
            return pack(pb + L.lm_off, m, cfg->vocab, L.lm.Nt * 16, 0, MAP_IDENT);
        }
    }
}

int card_verify(const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv, int32_t ctx_len,
                const int32_t* cand_tokens_dev, int32_t r, void* workspace_dev, void* stream,
                card_verify_result* out_dev, int32_t* row_argmax_dev) {
    return verify_impl(cfg, packed_weights_dev, kv, ctx_len, cand_tokens_dev, r, workspace_dev, stream, out_dev,
                       row_argmax_dev, nullptr);
}

int card_verify_sampled(const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv, int32_t ctx_len,
                        const int32_t* cand_tokens_dev, int32_t r, const card_sampling* sampling, void* workspace_dev,
                        void* stream, card_verify_result* out_dev, int32_t* row_token_dev, float* logits_dev) {
    if (!sampling || !(sampling->temperature >= 0.f)) return CARD_EINVAL;
    return verify_impl(cfg, packed_weights_dev, kv, ctx_len, cand_tokens_dev, r, workspace_dev, stream, out_dev,
                       row_token_dev, logits_dev, sampling);
}

int card_draft_level(const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv, int32_t ctx_len,
                     const card_tree_rows* rows, int32_t n_rows, int32_t k, void* workspace_dev, void* stream,
                     int32_t* topk_tokens_dev, float* topk_probs_dev, float* logits_dev) {
    if (!rows) return CARD_EINVAL;
    TreeOpt t = {rows->positions_dev, rows->first_slot, rows->mask_dev, rows->mask_words, rows->mask_base, k,
                 topk_tokens_dev, topk_probs_dev};
    card_kv kv2;
    if (!kv) return CARD_EINVAL;
    kv2 = *kv;
    kv2.pending_token = -1;
    return verify_impl(cfg, packed_weights_dev, &kv2, ctx_len, rows->tokens_dev, n_rows, workspace_dev, stream, nullptr,
                       nullptr, logits_dev, nullptr, &t);
}

int card_tree_mask_level(const uint32_t* parent_mask_host, const int32_t* parent_idx_host, int32_t n_rows,
                         int32_t first_slot, int32_t ctx_len, int32_t mask_base, int32_t mask_words,
                         uint32_t* out_mask_host) {
    if (!parent_idx_host || !out_mask_host || n_rows < 1) return CARD_EINVAL;
    if (mask_words < 1 || mask_words > 32 || mask_base < 0 || mask_base % kKvBlock || mask_base > ctx_len) return CARD_EINVAL;
    if (first_slot < ctx_len || int64_t(first_slot) + n_rows > int64_t(mask_base) + 32 * mask_words) return CARD_ERANGE;
    for (int i = 0; i < n_rows; ++i) {
        uint32_t* row = out_mask_host + size_t(i) * mask_words;
        const int p = parent_idx_host[i];
        if (p >= 0) {
            if (!parent_mask_host) return CARD_EINVAL;
            // inherit the parent's causal history
            for (int w = 0; w < mask_words; ++w) row[w] = parent_mask_host[size_t(p) * mask_words + w];
        } else {
            // a root of the tree sees the committed context only
            for (int w = 0; w < mask_words; ++w) row[w] = 0u;
            for (int s = mask_base; s < ctx_len; ++s) row[(s - mask_base) >> 5] |= 1u << ((s - mask_base) & 31);
        }
        const int own = first_slot + i - mask_base;  // ... plus the node itself; peers stay invisible
        row[own >> 5] |= 1u << (own & 31);
    }
    return CARD_OK;
}

int card_cache_select(const float* sigma_dev, const int32_t* topk_tokens_dev, const float* topk_probs_dev, int32_t n_parents,
                      int32_t k, int32_t K, int32_t* out_tokens_dev, float* out_scores_dev, int32_t* out_parents_dev,
                      void* stream) {
    if (!sigma_dev || !topk_tokens_dev || !topk_probs_dev || !out_tokens_dev || !out_scores_dev || !out_parents_dev)
        return CARD_EINVAL;
    if (n_parents < 1 || k < 1 || k > 16 || K < 1 || int64_t(n_parents) * k > 256 * kSelPerThread) return CARD_ERANGE;
    SelectArgs a = {sigma_dev, topk_tokens_dev, topk_probs_dev, n_parents, k, K, out_tokens_dev, out_scores_dev,
                    out_parents_dev};
    hipLaunchKernelGGL(k_cache_select, dim3(1), dim3(256), 0, as_stream(stream), a);
    const int st = launch_status();
    return st != CARD_OK ? st : (K < n_parents * k ? K : n_parents * k);
}

static int step_begin_impl(card_cache* cache, const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv,
                    int32_t ctx_len, int32_t max_len, int32_t* cand_staging, void* workspace_dev, void* stream,
                    card_verify_result* out, int32_t* row_argmax_dev, card_step* step_host, const card_sampling* sampling) {
    if (!cache || !cfg || !kv || !cand_staging || !step_host) return CARD_EINVAL;
    if (max_len < 1 || max_len > cfg->max_r || max_len > kMaxR) return CARD_ERANGE;
    if (kv->pending_token < 0) return CARD_EINVAL;  // the query key is the token just verified
    int32_t n = 0;
    float score = 0.f;
    const int hit = card_cache_query(cache, kv->pending_token, max_len, step_host->cand, &n, &score);
    if (hit < 0) return hit;
    if (hit == 0 || n < 1) {  // miss: a plain decode step on the verified token
        n = 1;
        step_host->cand[0] = kv->pending_token;
    }
    step_host->hit = hit > 0 ? 1 : 0;
    step_host->r = n;
    step_host->path_score = hit > 0 ? score : 0.f;
    for (int i = 0; i < n; ++i) cand_staging[i] = step_host->cand[i];
    return verify_impl(cfg, packed_weights_dev, kv, ctx_len, cand_staging, n, workspace_dev, stream, out, row_argmax_dev,
                       nullptr, sampling);
}


int card_step_begin(card_cache* cache, const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv,
                    int32_t ctx_len, int32_t max_len, int32_t* cand_staging, void* workspace_dev, void* stream,
                    card_verify_result* out, int32_t* row_argmax_dev, card_step* step_host) {
    return step_begin_impl(cache, cfg, packed_weights_dev, kv, ctx_len, max_len, cand_staging, workspace_dev, stream, out,
                           row_argmax_dev, step_host, nullptr);
}

int card_step_begin_sampled(card_cache* cache, const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv,
                    int32_t ctx_len, int32_t max_len, int32_t* cand_staging, void* workspace_dev, void* stream,
                    card_verify_result* out, int32_t* row_argmax_dev, card_step* step_host,
                            const card_sampling* sampling) {
    if (!sampling || !(sampling->temperature >= 0.f)) return CARD_EINVAL;
    return step_begin_impl(cache, cfg, packed_weights_dev, kv, ctx_len, max_len, cand_staging, workspace_dev, stream, out,
                           row_argmax_dev, step_host, sampling);
}

int card_step_end(card_cache* cache, const card_step* step_host, const card_verify_result* out_host, int32_t flags,
                  int32_t* emitted_host, int32_t* n_emitted_host) {
    if (!cache || !step_host || !out_host || !emitted_host || !n_emitted_host) return CARD_EINVAL;
    const int a = out_host->accepted_len;
    if (a < 1 || a > step_host->r) return CARD_EDEVICE;  // the step failed (or was not a CARD step)
    // what the step has verified beyond the query key: the accepted part of the path, then the target's own token
    int n = 0;
    for (int i = 1; i < a; ++i) emitted_host[n++] = step_host->cand[i];
    emitted_host[n++] = out_host->correction_token;
    *n_emitted_host = n;
    if (flags & CARD_STEP_NO_CORRECT) return CARD_OK;
    // the accepted candidates (query key first) are walked down the tree: the children of the last
    // one become level 0, where the next query looks the target's own token up
    const int st = card_cache_correct(cache, step_host->cand, a);
    return st < 0 ? st : CARD_OK;
}

int card_verify_static(const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv, int32_t ctx_len,
                       const int32_t* cand_tokens_dev, int32_t r, void* stream, card_verify_result* out_dev,
                       int32_t* row_argmax_dev) {
    const Layout L = make_layout(cfg);
    if (!L.ok || !packed_weights_dev || !kv || !cand_tokens_dev || !out_dev) return CARD_EINVAL;
    if (L.ws_bytes > kStaticWsBytes) return CARD_ETOOBIG;
    if (r < 1 || r > cfg->max_r) return CARD_ERANGE;  // nothing is enqueued for a call that will be refused
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CARD_EDEVICE;
    void* ws = nullptr;
    {
        std::lock_guard<std::mutex> g(g_static_mu);
        StaticWs& sw = g_static[dev];
        if (!sw.ptr) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CARD_EDEVICE;
            sw.ptr = p;
        }
        // The layout of the control words depends on the model: a call for another model than the
        // last one (or the first call) clears the part it uses and sets the mark, stream-ordered in
        // front of the step.  The array keeps the last call's contents otherwise.
        if (!sw.prepared || memcmp(&sw.cfg, cfg, sizeof(card_model_cfg)) != 0) {
            hipLaunchKernelGGL(k_ws_init, dim3(1024), dim3(256), 0, as_stream(stream), static_cast<uint4v*>(sw.ptr),
                               L.ws_bytes / 16, reinterpret_cast<uint32_t*>(static_cast<char*>(sw.ptr) + L.m_bar_off) + kBarMagic);
            if (launch_status() != CARD_OK) return CARD_EDEVICE;
            sw.cfg = *cfg;
            sw.prepared = true;
        }
        ws = sw.ptr;
    }
    return verify_impl(cfg, packed_weights_dev, kv, ctx_len, cand_tokens_dev, r, ws, stream, out_dev, row_argmax_dev,
                       nullptr);
}

size_t card_static_scratch_bytes(void) { return kStaticWsBytes; }

int card_static_scratch_reset(void) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CARD_EDEVICE;
    std::lock_guard<std::mutex> g(g_static_mu);
    g_static[dev].prepared = false;
    return CARD_OK;
}

int card_verify_debug_logits(const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv,
                             int32_t ctx_len, const int32_t* cand_tokens_dev, int32_t r, void* workspace_dev,
                             void* stream, card_verify_result* out_dev, int32_t* row_argmax_dev,
                             float* logits_dev) {
    if (!logits_dev) return CARD_EINVAL;
    return verify_impl(cfg, packed_weights_dev, kv, ctx_len, cand_tokens_dev, r, workspace_dev, stream, out_dev,
                       row_argmax_dev, logits_dev);
}

int card_profile_timeline(void* buf_dev, int32_t layer) {
    g_ts_buf = static_cast<unsigned long long*>(buf_dev);
    g_ts_layer = layer;
    return CARD_OK;
}

int card_profile_enable(int32_t max_launches) {
    if (max_launches <= 0) return CARD_EINVAL;
    Profile& p = prof();
    std::lock_guard<std::mutex> g(p.mu);
    while (int(p.start.size()) < max_launches) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return CARD_EDEVICE;
        if (hipEventCreate(&b) != hipSuccess) {
            (void)hipEventDestroy(a);
            return CARD_EDEVICE;
        }
        p.start.push_back(a);
        p.stop.push_back(b);
    }
    p.used = 0;
    p.on = true;
    return CARD_OK;
}

int card_profile_collect(float* ms_host, int32_t* n_host) {
    if (!ms_host || !n_host) return CARD_EINVAL;
    Profile& p = prof();
    std::lock_guard<std::mutex> g(p.mu);
    const int n = p.used;
    p.on = false;
    p.used = 0;
    for (int i = 0; i < n; ++i) {
        if (hipEventSynchronize(p.stop[i]) != hipSuccess) return CARD_EDEVICE;
        if (hipEventElapsedTime(&ms_host[i], p.start[i], p.stop[i]) != hipSuccess) return CARD_EDEVICE;
    }
    *n_host = n;
    return CARD_OK;
}

int card_profile_disable(void) {
    Profile& p = prof();
    std::lock_guard<std::mutex> g(p.mu);
    p.on = false;
    p.used = 0;
    int st = CARD_OK;
    for (hipEvent_t e : p.start)
        if (hipEventDestroy(e) != hipSuccess) st = CARD_EDEVICE;
    for (hipEvent_t e : p.stop)
        if (hipEventDestroy(e) != hipSuccess) st = CARD_EDEVICE;
    p.start.clear();
    p.stop.clear();
    return st;
}

int card_workspace_init(const card_model_cfg* cfg, void* workspace_dev, void* stream) {
    if (!workspace_dev) return CARD_EINVAL;
    const Layout L = make_layout(cfg);
    if (!L.ok) return CARD_EINVAL;
    char* ws = static_cast<char*>(workspace_dev);
    if (reinterpret_cast<uintptr_t>(ws) % 16 || L.ws_bytes % 16) return CARD_EINVAL;
    hipLaunchKernelGGL(k_ws_init, dim3(1024), dim3(256), 0, as_stream(stream), reinterpret_cast<uint4v*>(ws),
                       L.ws_bytes / 16, reinterpret_cast<uint32_t*>(ws + L.m_bar_off) + kBarMagic);
    return launch_status();
}

int card_kv_gather(const card_model_cfg* cfg, const card_kv* kv, int32_t layer, int32_t first_slot, int32_t count,
                   float* k_out_dev, float* v_out_dev, void* stream) {
    if (!cfg_valid(cfg) || !kv || !kv->k_pages || !kv->v_pages || !kv->block_table || !k_out_dev || !v_out_dev)
        return CARD_EINVAL;
    if (layer < 0 || layer >= cfg->n_layers || count <= 0 || first_slot < 0) return CARD_ERANGE;
    if (int64_t(first_slot) + count > cfg->max_ctx) return CARD_ECAPACITY;
    const size_t pool_layer_elems = size_t(kv->n_pages) * cfg->n_kv_heads * 16 * cfg->head_dim;
    GatherArgs a = {};
    a.kpool = static_cast<const __bf16*>(kv->k_pages) + size_t(layer) * pool_layer_elems;
    a.vpool = static_cast<const __bf16*>(kv->v_pages) + size_t(layer) * pool_layer_elems;
    a.block_table = kv->block_table;
    a.first = first_slot;
    a.count = count;
    a.n_kv_heads = cfg->n_kv_heads;
    a.head_dim = cfg->head_dim;
    a.k_out = k_out_dev;
    a.v_out = v_out_dev;
    const int64_t total = int64_t(count) * cfg->n_kv_heads * cfg->head_dim;
    hipLaunchKernelGGL(k_kv_gather, dim3(uint32_t((total + 255) / 256)), dim3(256), 0, as_stream(stream), a);
    return launch_status();
}

}  // extern "C"
