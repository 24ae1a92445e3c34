// C ABI of libcard: argument checks and the launch sequence of one verification step.
#include <hip/hip_runtime.h>

#include <vector>

#include "card.h"
#include "card_kernels.hip"
#include "card_mega.hip"

using namespace card;

namespace {

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

inline int launch_status() { return hipGetLastError() == hipSuccess ? CARD_OK : CARD_EDEVICE; }

unsigned long long* g_ts_buf = nullptr;
int g_ts_layer = 0;
bool g_use_mega = true;  // TEMPORARY while the persistent kernel is brought up

// benchmark hook: event pairs around one kernel kind
struct Profile {
    int kind = -1;
    int used = 0;
    std::vector<hipEvent_t> start, stop;
};
Profile g_prof;

struct ProfScope {
    hipStream_t st;
    int idx = -1;
    ProfScope(int kind, hipStream_t s) : st(s) {
        if (g_prof.kind == kind && g_prof.used < int(g_prof.start.size())) {
            idx = g_prof.used++;
            (void)hipEventRecord(g_prof.start[idx], st);
        }
    }
    ~ProfScope() {
        if (idx >= 0) (void)hipEventRecord(g_prof.stop[idx], st);
    }
};

template <int MT>
int launch_gemm(int epi, const GemmArgs& a, const GemmPlan& p, hipStream_t st) {
    const dim3 grid(p.groups * p.splits), block(kGemmWaves * 64);
    switch (epi) {
        case EPI_QKV: hipLaunchKernelGGL((k_gemm<MT, EPI_QKV>), grid, block, 0, st, a); break;
        case EPI_RESID: hipLaunchKernelGGL((k_gemm<MT, EPI_RESID>), grid, block, 0, st, a); break;
        case EPI_SWIGLU: hipLaunchKernelGGL((k_gemm<MT, EPI_SWIGLU>), grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL((k_gemm<MT, EPI_LMHEAD>), grid, block, 0, st, a); break;
    }
    return launch_status();
}

int gemm(int epi, int r, const GemmArgs& a, const GemmPlan& p, hipStream_t st) {
    return r <= 16 ? launch_gemm<1>(epi, a, p, st) : launch_gemm<2>(epi, a, p, st);
}

GemmArgs base_args(const char* wbase, const MatDesc& m, const GemmPlan& p, const float* xin, int ldx, int r,
                   char* ws, const Layout& L) {
    GemmArgs a = {};
    a.w = reinterpret_cast<const bf16x8*>(wbase + m.off);
    a.N = m.N;
    a.K = m.K;
    a.Nt = m.Nt;
    a.Ks = m.Ks;
    a.splits = p.splits;
    a.steps_per_split = p.steps_per_split;
    a.xin = xin;
    a.ldx = ldx;
    a.r = r;
    a.part = reinterpret_cast<float*>(ws + L.part_off);
    a.counters = reinterpret_cast<int32_t*>(ws + L.cnt_off);
    return a;
}

int cu_count() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cus = n;
    }
    return cus;
}

template <int MT, int H>
int launch_mega(MegaArgs& a, hipStream_t st) {
    void* params[] = {&a};
    const hipError_t e = hipLaunchCooperativeKernel(reinterpret_cast<void*>(k_verify<MT, H>), dim3(a.nwg),
                                                    dim3(kMegaThreads), params, 0, st);
    return e == hipSuccess ? CARD_OK : CARD_EDEVICE;
}

// One persistent cooperative kernel runs the whole step.
int verify_mega(const card_model_cfg* cfg, const void* packed, const card_kv* kv, int32_t ctx_len,
                const int32_t* cand, int32_t r, void* workspace, void* stream, card_verify_result* out,
                int32_t* row_argmax, float* logits) {
    if (!cfg || !packed || !kv || !cand || !workspace || !out) return CARD_EINVAL;
    const Layout L = make_layout(cfg);
    if (!L.ok) return CARD_EINVAL;
    if (!kv->k_pages || !kv->v_pages || !kv->block_table || kv->n_pages <= 0) return CARD_EINVAL;
    if (r < 1 || r > cfg->max_r) return CARD_ERANGE;
    if (ctx_len < 0) return CARD_EINVAL;
    if (int64_t(ctx_len) + r > cfg->max_ctx) return CARD_ECAPACITY;
    int cus = cu_count();
    if (cus <= 0) return CARD_EDEVICE;
    if (cus > 256) cus = 256;  // the barrier polls at most 256 flag words

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
    a.inv_sqrt_h = 1.0f / sqrtf(float(h));
    a.wbase = static_cast<const char*>(packed);
    a.embed_off = L.embed_off;
    a.g_final_off = L.g_final_off;
    a.layer0_off = L.layer0_off;
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
    a.pages_used = ceil_div(ctx_len + r, kKvBlock);
    a.row_tiles = ceil_div(a.G * r, 16);
    // cut the context only when a wavefront would walk more than ten pages (pages are pulled into
    // the near cache ahead of time, so a short walk is cheaper than merging cuts)
    int splits = ceil_div(a.pages_used, 10 * kMegaWaves);
    if (splits > L.m_attn_max_splits) splits = L.m_attn_max_splits;
    a.pages_per_split = ceil_div(a.pages_used, splits);
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
    a.flags = reinterpret_cast<uint32_t*>(ws + L.m_flags_off);
    a.cand = cand;
    a.pending = kv->pending_token;
    a.out = out;
    a.row_argmax = row_argmax;
    a.logits = logits;
    a.ts = g_ts_buf;
    a.ts_layer = g_ts_layer;
    hipStream_t st = as_stream(stream);
    ProfScope ps(CARD_K_STEP, st);
    if (r <= 16) return h == 128 ? launch_mega<1, 128>(a, st) : launch_mega<1, 64>(a, st);
    return h == 128 ? launch_mega<2, 128>(a, st) : launch_mega<2, 64>(a, st);
}

int verify_impl(const card_model_cfg* cfg, const void* packed, const card_kv* kv, int32_t ctx_len,
                const int32_t* cand, int32_t r, void* workspace, void* stream, card_verify_result* out,
                int32_t* row_argmax, float* logits) {
    if (!cfg || !packed || !kv || !cand || !workspace || !out) return CARD_EINVAL;
    const Layout L = make_layout(cfg);
    if (!L.ok) return CARD_EINVAL;
    if (!kv->k_pages || !kv->v_pages || !kv->block_table || kv->n_pages <= 0) return CARD_EINVAL;
    if (r < 1 || r > cfg->max_r) return CARD_ERANGE;
    if (ctx_len < 0) return CARD_EINVAL;
    if (int64_t(ctx_len) + r > cfg->max_ctx) return CARD_ECAPACITY;

    hipStream_t st = as_stream(stream);
    const char* wb = static_cast<const char*>(packed);
    char* ws = static_cast<char*>(workspace);
    const int d = cfg->d_model, h = cfg->head_dim, qd = cfg->n_q_heads * h, kvd = cfg->n_kv_heads * h;
    const int G = cfg->n_q_heads / cfg->n_kv_heads;
    float* x = reinterpret_cast<float*>(ws + L.x_off);
    float* q = reinterpret_cast<float*>(ws + L.q_off);
    float* att = reinterpret_cast<float*>(ws + L.att_off);
    float* act = reinterpret_cast<float*>(ws + L.act_off);
    float* ss = reinterpret_cast<float*>(ws + L.ss_off);
    float* rope = reinterpret_cast<float*>(ws + L.rope_off);
    int32_t* acnt = reinterpret_cast<int32_t*>(ws + L.acnt_off);
    const float inv_d = 1.0f / float(d);

    // attention decomposition
    const int row_tiles = ceil_div(G * r, 16), row_pairs = ceil_div(row_tiles, 2);
    const int pages_used = ceil_div(ctx_len + r, kKvBlock);
    int a_splits = ceil_div(256, cfg->n_kv_heads * row_pairs);
    const int max_by_pages = ceil_div(pages_used, kAttnWaves);
    if (a_splits > max_by_pages) a_splits = max_by_pages;
    if (a_splits > L.attn_max_splits) a_splits = L.attn_max_splits;
    if (a_splits < 1) a_splits = 1;
    const int pages_per_split = ceil_div(pages_used, a_splits);
    a_splits = ceil_div(pages_used, pages_per_split);

    {
        EmbedArgs e = {};
        e.embed = reinterpret_cast<const __bf16*>(wb + L.embed_off);
        e.tokens = cand;
        e.r = r;
        e.d = d;
        e.vocab = cfg->vocab;
        e.x = x;
        e.ss_out = ss;
        e.rope = rope;
        e.ctx_len = ctx_len;
        e.head_dim = h;
        e.theta = cfg->rope_theta;
        e.counters = reinterpret_cast<int32_t*>(ws + L.cnt_off);
        e.n_counters = L.n_counters;
        e.acounters = acnt;
        e.n_acounters = cfg->n_kv_heads * ceil_div(L.attn_row_tiles_max, 2);
        e.best = reinterpret_cast<unsigned long long*>(ws + L.best_off);
        hipLaunchKernelGGL(k_embed, dim3(d / 64), dim3(64), 0, st, e);
        if (launch_status() != CARD_OK) return CARD_EDEVICE;
    }

    const size_t pool_layer_elems = size_t(kv->n_pages) * cfg->n_kv_heads * 16 * h;
    for (int l = 0; l < cfg->n_layers; ++l) {
        const char* lb = wb + L.layer0_off + size_t(l) * L.layer_stride;
        __bf16* kpool = static_cast<__bf16*>(kv->k_pages) + size_t(l) * pool_layer_elems;
        __bf16* vpool = static_cast<__bf16*>(kv->v_pages) + size_t(l) * pool_layer_elems;
        {
            GemmArgs a = base_args(lb, L.qkv, L.p_qkv, x, d, r, ws, L);
            a.gain = reinterpret_cast<const float*>(lb + L.g_attn_off);
            a.ss_in = ss;
            a.ss_in_groups = L.ss_groups;
            a.inv_d = inv_d;
            a.eps = cfg->rms_eps;
            a.q = q;
            a.kpool = kpool;
            a.vpool = vpool;
            a.block_table = kv->block_table;
            a.rope = rope;
            a.ctx_len = ctx_len;
            a.head_dim = h;
            a.q_dim = qd;
            a.kv_dim = kvd;
            a.n_kv_heads = cfg->n_kv_heads;
            ProfScope ps(CARD_K_QKV, st);
            if (gemm(EPI_QKV, r, a, L.p_qkv, st) != CARD_OK) return CARD_EDEVICE;
        }
        {
            AttnArgs a = {};
            a.q = q;
            a.kpool = kpool;
            a.vpool = vpool;
            a.block_table = kv->block_table;
            a.r = r;
            a.G = G;
            a.n_kv_heads = cfg->n_kv_heads;
            a.q_dim = qd;
            a.ctx_len = ctx_len;
            a.n_pages_used = pages_used;
            a.splits = a_splits;
            a.pages_per_split = pages_per_split;
            a.row_pairs = row_pairs;
            a.inv_sqrt_h = 1.0f / sqrtf(float(h));
            a.part = reinterpret_cast<float*>(ws + L.apart_off);
            a.counters = acnt;
            a.att = att;
            ProfScope ps(CARD_K_ATTN, st);
            const dim3 grid(cfg->n_kv_heads * row_pairs * a_splits), block(kAttnWaves * 64);
            if (h == 128)
                hipLaunchKernelGGL(k_attn<128>, grid, block, 0, st, a);
            else
                hipLaunchKernelGGL(k_attn<64>, grid, block, 0, st, a);
            if (launch_status() != CARD_OK) return CARD_EDEVICE;
        }
        {
            GemmArgs a = base_args(lb, L.wo, L.p_wo, att, qd, r, ws, L);
            a.x = x;
            a.ss_out = ss;
            ProfScope ps(CARD_K_WO, st);
            if (gemm(EPI_RESID, r, a, L.p_wo, st) != CARD_OK) return CARD_EDEVICE;
        }
        {
            GemmArgs a = base_args(lb, L.gu, L.p_gu, x, d, r, ws, L);
            a.gain = reinterpret_cast<const float*>(lb + L.g_ffn_off);
            a.ss_in = ss;
            a.ss_in_groups = L.ss_groups;
            a.inv_d = inv_d;
            a.eps = cfg->rms_eps;
            a.act = act;
            a.F = cfg->d_ffn;
            ProfScope ps(CARD_K_GATE_UP, st);
            if (gemm(EPI_SWIGLU, r, a, L.p_gu, st) != CARD_OK) return CARD_EDEVICE;
        }
        {
            GemmArgs a = base_args(lb, L.wd, L.p_wd, act, cfg->d_ffn, r, ws, L);
            a.x = x;
            a.ss_out = ss;
            ProfScope ps(CARD_K_DOWN, st);
            if (gemm(EPI_RESID, r, a, L.p_wd, st) != CARD_OK) return CARD_EDEVICE;
        }
    }
    {
        GemmArgs a = base_args(wb, L.lm, L.p_lm, x, d, r, ws, L);
        a.gain = reinterpret_cast<const float*>(wb + L.g_final_off);
        a.ss_in = ss;
        a.ss_in_groups = L.ss_groups;
        a.inv_d = inv_d;
        a.eps = cfg->rms_eps;
        a.best = reinterpret_cast<unsigned long long*>(ws + L.best_off);
        a.logits = logits;
        ProfScope ps(CARD_K_LM_HEAD, st);
        if (gemm(EPI_LMHEAD, r, a, L.p_lm, st) != CARD_OK) return CARD_EDEVICE;
    }
    {
        AcceptArgs a = {};
        a.best = reinterpret_cast<const unsigned long long*>(ws + L.best_off);
        a.r = r;
        a.cand = cand;
        a.pending = kv->pending_token;
        a.ctx_len = ctx_len;
        a.out = out;
        a.row_argmax = row_argmax;
        hipLaunchKernelGGL(k_accept, dim3(1), dim3(64), 0, st, a);
        if (launch_status() != CARD_OK) return CARD_EDEVICE;
    }
    return CARD_OK;
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
    return (g_use_mega ? verify_mega : verify_impl)(cfg, packed_weights_dev, kv, ctx_len, cand_tokens_dev, r,
                                                    workspace_dev, stream, out_dev, row_argmax_dev, nullptr);
}

int card_verify_debug_logits(const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv,
                             int32_t ctx_len, const int32_t* cand_tokens_dev, int32_t r, void* workspace_dev,
                             void* stream, card_verify_result* out_dev, int32_t* row_argmax_dev,
                             float* logits_dev) {
    if (!logits_dev) return CARD_EINVAL;
    return (g_use_mega ? verify_mega : verify_impl)(cfg, packed_weights_dev, kv, ctx_len, cand_tokens_dev, r,
                                                    workspace_dev, stream, out_dev, row_argmax_dev, logits_dev);
}

int card_debug_timeline(void* buf_dev, int32_t layer) {
    g_ts_buf = static_cast<unsigned long long*>(buf_dev);
    g_ts_layer = layer;
    return CARD_OK;
}

int card_debug_use_mega(int on) {
    g_use_mega = on != 0;
    return CARD_OK;
}

int card_profile_enable(int32_t kind, int32_t max_launches) {
    if (kind < CARD_K_QKV || kind > CARD_K_STEP || max_launches <= 0) return CARD_EINVAL;
    while (int(g_prof.start.size()) < max_launches) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return CARD_EDEVICE;
        g_prof.start.push_back(a);
        g_prof.stop.push_back(b);
    }
    g_prof.kind = kind;
    g_prof.used = 0;
    return CARD_OK;
}

int card_profile_collect(float* ms_host, int32_t* n_host) {
    if (!ms_host || !n_host) return CARD_EINVAL;
    const int n = g_prof.used;
    g_prof.kind = -1;
    g_prof.used = 0;
    for (int i = 0; i < n; ++i) {
        if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess) return CARD_EDEVICE;
        if (hipEventElapsedTime(&ms_host[i], g_prof.start[i], g_prof.stop[i]) != hipSuccess) return CARD_EDEVICE;
    }
    *n_host = n;
    return CARD_OK;
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
