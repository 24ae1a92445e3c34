// The whole verification step as ONE persistent kernel (one workgroup per compute unit).
//
// Why: at r <= 32 rows a decoder layer is five dependent, HBM-bound phases of 4-30 us each,
// separated by hand-overs of (tiny) activations that cost several microseconds of pure latency
// each (store acknowledgement, barrier, first touch of the new activations).  Weights never
// depend on activations, so the kernel decouples the two:
//
//   * four PRODUCER wavefronts per workgroup (one per SIMD) walk the workgroup's weight
//     fragments of the whole step in consumption order, keep 8 loads of 1 KiB in flight each
//     and push what arrives into a per-wavefront FIFO in LDS (28 KiB each).  The weights are
//     stored in exactly that order, so each producer reads one contiguous run per matrix (four
//     interleaved runs in the grouped down-projection of the kernels for r > 8: plan_phase_grouped);
//   * four CONSUMER wavefronts pop fragments from their FIFO into the matrix pipe, run the
//     epilogues, the attention phase and the grid barriers.
//
// The producers never wait for a barrier, only for FIFO space: HBM keeps streaming through
// every hand-over until 36 KiB per wavefront pair (37 MB on the whole part) are buffered, and
// the consumers catch up from LDS afterwards.
//
// Hand-over rules (the part has one L2 per compute die, not coherent with the others):
//   * everything one workgroup writes for another is stored with device scope (write-through);
//   * every such buffer is written exactly once per call, at an address nobody has read before
//     in this call (one copy per layer and phase), so plain cached loads can never hit a stale
//     line; the barrier flags themselves are only touched with device-scope accesses.
//
// Activations travel between phases already split into bf16 high + low halves and laid out in
// the operand order of the matrix instruction ("fragment order"): element (row m, column k) of
// an r x K activation lives at ((k/8) * rp + m) * 16 + k%8 (high half) and +8 (low half), where
// rp = r rounded up to 8.  A wavefront's operand load for one 32-deep k-step is then one
// contiguous rp*128-byte run.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "card_common.hip"

namespace card {


typedef __attribute__((ext_vector_type(2))) unsigned int uint2v;

constexpr int kMegaWaves = 4;             // consumer wavefronts, one per SIMD (they cut K four ways)
constexpr int kMegaThreads = kMegaWaves * 64;
static_assert(kMegaWaves == kStreamWaves, "the weight layout assumes this many wavefront pairs");
constexpr int kProdWaves = kMegaWaves;    // producer wavefront p feeds consumer wavefront p
constexpr int kBlockThreads = (kMegaWaves + kProdWaves) * 64;
constexpr int kRing = 8;                 // weight fragments (1 KiB each) in flight per producer
constexpr int kFifo = 28;                 // fragment slots per FIFO
constexpr int kGroup = 8;                 // fragments a consumer pops at a time (SG k-steps x NB tiles)
constexpr uint32_t kSpinLimit = 1u << 20; // bounded barrier wait: the kernel always terminates
constexpr uint32_t kLdsSpinLimit = 1u << 24;  // bounded FIFO waits (each poll is an LDS round trip)

struct MegaArgs {
    int32_t L, d, qd, kvd, h, Hkv, G, F, V, r, rp, ctx_len, nwg;
    float eps, inv_d, theta, inv_sqrt_h;
    const char* wbase;
    const uint32_t* stamp;  // {magic, grid size} the weights were laid out for
    size_t embed_off, g_final_off, layer0_off, layer_stride, g_attn_off, g_ffn_off;
    MatDesc qkv, wo, gu, wd, lm;  // lm.off absolute, the others relative to the layer base
    __bf16* kpool;
    __bf16* vpool;
    size_t pool_layer_elems;
    const int32_t* block_table;
    int32_t pages_used, a_splits, pages_per_split, row_tiles;
    // workspace; "v" = residual version: 0 after embed, 2l+1 after O-proj, 2l+2 after down of layer l
    float* xres;       // [2L+1][32][d]
    __bf16* xfrag;     // [2L+1][xfrag_stride]
    float* ss;         // [2L+1][32][d/16]
    __bf16* qfrag;     // [L][Hkv][G*32][h/8][16]
    __bf16* attfrag;   // [L][attfrag_stride]
    __bf16* actfrag;   // [L][actfrag_stride]
    float* apart;      // [tasks][16*(h+2)], shared by all layers (read back with device-scope loads)
    size_t xfrag_stride, attfrag_stride, actfrag_stride, qfrag_stride;
    float* rope;
    unsigned long long* best;
    uint32_t* bar;     // kBarExit, kBarError (zero between calls), kBarEpoch, kBarMagic
    uint32_t* flags;   // [kFlagCopies][256] last barrier sequence number each workgroup has reached
    uint32_t* acount;  // [Hkv * row_tiles] arrival counters of the attention cuts; zero between uses
    float* dpart;      // [d/16 tiles][4 quarters of K][16][32] partial down-projection blocks (r > 8)
    uint32_t* dcount;  // [d/64] arrival counters of the groups of four tiles; zero between uses
    const int32_t* cand;
    // draft-side tree rows (all zero / null for a verification step): row m sits at sequence position
    // row_pos[m] and in cache slot slot0 + m; it sees every slot below tmask_base and, from there on,
    // the slots whose bit is set in its mask row tmask[m * tmask_words ..]
    int32_t slot0, old_end;       // slot of row 0; slots below old_end hold context written by earlier calls
    const int32_t* row_pos;
    const uint32_t* tmask;
    int32_t tmask_words, tmask_base;
    // per-row top-k of the vocabulary phase instead of the arg-max (topk = 0: arg-max)
    int32_t topk;
    unsigned long long* topk_part;  // [nwg][kMaxR][16] best keys of each workgroup's columns
    float* lse_part;                // [nwg][kMaxR][2]  (max, sum of exp) of each workgroup's columns
    int32_t* topk_tok;              // out [r][topk]
    float* topk_prob;               // out [r][topk]
    int32_t pending;
    float inv_temp;          // 0: greedy (arg-max of the logits); > 0: sample, logits / temperature + Gumbel noise
    uint32_t seed_lo, seed_hi;
    card_verify_result* out;
    int32_t* row_argmax;
    float* logits;
    unsigned long long* ts;  // optional phase timeline [nwg][32] of layer ts_layer (100 MHz ticks)
    int32_t ts_layer;
};

struct __align__(16) MegaSmem {
    uint4v fifo[kMegaWaves][kFifo][64];               // weight fragments, producer -> consumer
    union {
        float red[kMegaWaves * 8 * 256];              // GEMM: per-wavefront accumulators (after the k-loop)
        float attn[kMegaWaves * 16 * (128 + 2)];      // attention: per-wavefront (M, L, O)
    };
    float tile[2048];        // reduced outputs of one batch: [NB*16 rows][16*MT columns]
    float row_scale[kMaxR];
    float wgt[(kMegaWaves + 3) * 16];
    unsigned long long part_best[512];
    unsigned long long wg_best[kMaxR];
    uint4v dump[64];             // where a producer writes ring slots that hold no fragment (end of the stream)
    uint32_t tail[kMegaWaves];   // fragments pushed so far (written by the producer)
    uint32_t head[kMegaWaves];   // fragments popped so far (written by the consumer)
    uint32_t cbar;               // arrivals at the consumer barrier (monotonic)
    int failed;
    int ws_ok;
    uint32_t epoch;
    int pred[kMaxR + 1];
};

// ---- device-scope (write-through) stores -------------------------------------------------
// 128-bit buffer stores with the device-scope bit: `ubase` is wavefront-uniform, `off` the
// lane's byte offset from it (< 4 GiB).
constexpr int kAuxDev = 16;  // sc1: device scope
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ void st_dev_b128(const void* ubase, uint32_t off, uint4v v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, make_rsrc(ubase, 0xffffffffu), int(off), 0, kAuxDev);
}
__device__ __forceinline__ void st_dev_f32x8(const float* ubase, uint32_t elem_off, const float (&v)[8]) {
    st_dev_b128(ubase, elem_off * 4, uint4v{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]),
                                             __float_as_uint(v[3])});
    st_dev_b128(ubase, elem_off * 4 + 16, uint4v{__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]),
                                                  __float_as_uint(v[7])});
}
__device__ __forceinline__ void st_dev_bf16(__bf16* p, __bf16 v) {
    __hip_atomic_store(reinterpret_cast<unsigned short*>(p), __builtin_bit_cast(unsigned short, v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t pack_bf16(__bf16 lo16, __bf16 hi16) {
    return uint32_t(__builtin_bit_cast(unsigned short, lo16)) | (uint32_t(__builtin_bit_cast(unsigned short, hi16)) << 16);
}
// eight values -> high and low bf16 halves -> 32 contiguous bytes at element offset `elem_off`
__device__ __forceinline__ void st_dev_frag8(const __bf16* ubase, size_t elem_off, const float (&v)[8]) {
    uint4v hi, lo;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        __bf16 h0, l0, h1, l1;
        split_bf16(v[e], h0, l0);
        split_bf16(v[e + 1], h1, l1);
        hi[e / 2] = pack_bf16(h0, h1);
        lo[e / 2] = pack_bf16(l0, l1);
    }
    st_dev_b128(ubase, uint32_t(elem_off * 2), hi);
    st_dev_b128(ubase, uint32_t(elem_off * 2) + 16, lo);
}
__device__ __forceinline__ size_t frag_index(int k, int m, int rp) { return (size_t(k >> 3) * rp + m) * 16 + (k & 7); }

// Values derived from the lane index are cheap to recompute but the optimiser likes to hoist
// them out of the layer loop, where dozens of them then stay live across every phase.  Passing
// the index through an empty asm at the top of each phase keeps them local to the phase.
__device__ __forceinline__ int opaque_v(int v) {
    asm volatile("" : "+v"(v));
    return v;
}

// ---- waits and barriers ------------------------------------------------------------------------
// All of this thread's global stores acknowledged.  (Consumer wavefronts have no long-latency
// loads queued: the weight stream belongs to the producers.)
__device__ __forceinline__ void store_wait() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));  // vmcnt(0)
}

// lgkmcnt(0) only: vmcnt(63) expcnt(7)
constexpr int kWaitLds = (63 & 15) | (7 << 4) | (0 << 8) | ((63 >> 4) << 14);

__device__ __forceinline__ uint32_t lds_peek(uint32_t* p) {
    return __builtin_amdgcn_readfirstlane(__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
}
__device__ __forceinline__ void lds_post(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Barrier of the four consumer wavefronts.  The hardware workgroup barrier would also wait for
// the producers, which never stop; this one is a monotonic arrival counter in LDS.  LDS executes
// one wavefront's instructions in order, so the arrival is performed after the wavefront's
// earlier LDS writes.  Every consumer wavefront executes the same sequence of these barriers.
__device__ __forceinline__ void cbar(MegaSmem& sm, uint32_t& cgen) {
    cgen += kMegaWaves;
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(kWaitLds);
    if ((threadIdx.x & 63) == 0) __hip_atomic_fetch_add(&sm.cbar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    while (int32_t(lds_peek(&sm.cbar) - cgen) < 0) __builtin_amdgcn_s_sleep(1);
    asm volatile("" ::: "memory");
}

// Grid barrier: arrive and wait.  A single counter would serialise one device-scope atomic per
// workgroup (about 10 us for 256 of them under load); instead every workgroup publishes the
// barrier's sequence number in its own flag word and consumer wavefront 0 of every workgroup
// polls all flags with one 1 KiB device-scope load.  Sequence numbers keep growing across calls
// (`epoch`), so flags never need clearing.  Callers have waited for their stores.
__device__ __forceinline__ void grid_wait(const MegaArgs& a, uint32_t& gen, MegaSmem& sm, uint32_t& cgen) {
    cbar(sm, cgen);
    gen += 1;
    if (threadIdx.x == 0 && sm.failed) {  // a bounded wait ran out in this workgroup: tell the one that reports
        __hip_atomic_store(&a.bar[kBarError], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));
    }
    if (threadIdx.x < 64 && !sm.failed) {
        const uint32_t target = sm.epoch + gen;
        const int lane = threadIdx.x;
        // every copy gets the flag; a workgroup polls the copy of its own residue class, so a
        // poll round puts 32 readers on a line instead of 256
        if (lane < kFlagCopies)
            __hip_atomic_store(&a.flags[lane * 256 + blockIdx.x], target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const __amdgpu_buffer_rsrc_t frs = make_rsrc(a.flags + (blockIdx.x % kFlagCopies) * 256, uint32_t(a.nwg) * 4);
        uint32_t spins = 0;
        while (true) {
            const uint4v f = __builtin_amdgcn_raw_buffer_load_b128(frs, lane * 16, 0, kAuxDev);
            bool ok = true;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (lane * 4 + q < a.nwg) ok = ok && int32_t(f[q] - target) >= 0;
            if (__builtin_amdgcn_ballot_w64(!ok) == 0ull) break;
            __builtin_amdgcn_s_sleep(1);
            if (++spins > kSpinLimit) {
                if (lane == 0) {
                    sm.failed = 1;
                    __hip_atomic_store(&a.bar[kBarError], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                break;
            }
        }
    }
    cbar(sm, cgen);
}

// ---- the weight stream -------------------------------------------------------------------------
// All streaming loads are buffer loads: a wavefront-uniform 128-bit resource (matrix base and
// size, in scalar registers), a wavefront-uniform 32-bit byte offset (scalar) and the lane's own
// 16-byte slot.
constexpr int kAuxNT = 2;  // non-temporal: weights are used once
constexpr int kOutOfRange = int(0x80000000u);  // lane offset beyond any buffer: the load returns 0, touches nothing

// One GEMM phase as seen by wavefront pair `wave` of workgroup `wg`: the workgroup's n-tiles are
// t_first + j * nwg (j < cnt), taken NB at a time ("batch"); the pair's k-steps are [s0, s1).
// The weights are stored in stream order (batch, then k-step, then tile of the batch): the pair's
// fragments of the phase are the cnt * (s1 - s0) KiB starting at byte `first` of the matrix.
struct PhasePlan {
    const bf16x8* w;
    uint32_t bytes, first;
    int32_t Ks, Nt, t_first, cnt, s0, s1;
    // grouped plan only (plan_phase_grouped): bytes from a tile's fragment to the next tile's of the
    // same k-step, bytes from one batch's first fragment to the next batch's, the workgroup's quarter
    uint32_t stride, batch_skip;
    int32_t quarter;
};

__device__ __forceinline__ PhasePlan plan_phase(const bf16x8* w, int Nt, int Ks, int wg, int nwg, int rot, int wave) {
    PhasePlan p;
    p.w = w;
    p.bytes = uint32_t(Nt) * uint32_t(Ks) * 1024u;
    p.Ks = Ks;
    p.Nt = Nt;
    p.t_first = (wg + rot) % nwg;
    const StreamRun r = stream_run(Nt, Ks, nwg, p.t_first, wave);
    p.cnt = r.cnt;
    p.s0 = r.s0;
    p.s1 = r.s1;
    p.first = uint32_t(r.first) << 10;
    p.stride = 0u;
    p.batch_skip = 0u;
    p.quarter = 0;
    return p;
}

// The same matrix, the same packed order, another division of the work, for phases in which a
// workgroup owns a single tile and r > 8: there every wavefront pulls r/8 KiB of activations
// through the vector L1 per KiB of weights, and that path, not HBM, sets the pace.  Four
// workgroups whose grid positions differ in the last two bits form a group and share the
// group's tiles (one per position and batch): position 4g + j takes the j-th quarter of K of
// all four tiles, its wavefront pair i the i-th quarter of that.  A wavefront then uses every
// activation operand for four tiles (a quarter of the L1 traffic per weight fragment), a pair
// streams four runs (one per tile, `stride` bytes apart) interleaved k-step by k-step, and the
// four workgroups' partial sums meet in memory.  Needs the four positions of a group to own
// equally many tiles: tile count and grid size multiples of four.
__device__ __forceinline__ PhasePlan plan_phase_grouped(const bf16x8* w, int Nt, int Ks, int wg, int nwg, int rot, int wave) {
    PhasePlan p;
    p.w = w;
    p.bytes = uint32_t(Nt) * uint32_t(Ks) * 1024u;
    p.Ks = Ks;
    p.Nt = Nt;
    const int pos = (wg + rot) % nwg, g0 = pos & ~3;
    p.quarter = pos & 3;
    const StreamRun q = stream_run(Nt, Ks, nwg, g0, p.quarter);  // the quarter's run of position g0
    const int len = q.s1 - q.s0;
    p.s0 = q.s0 + (wave * len) / kStreamWaves;
    p.s1 = q.s0 + ((wave + 1) * len) / kStreamWaves;
    p.t_first = g0;
    p.cnt = 4 * q.cnt;
    p.first = uint32_t(q.first + (p.s0 - q.s0)) << 10;
    p.stride = (uint32_t(q.cnt) * uint32_t(Ks)) << 10;  // a position's region of the matrix
    p.batch_skip = uint32_t(len) << 10;
    return p;
}

enum StreamPhase { SP_QKV = 0, SP_WO = 1, SP_GU = 2, SP_WD = 3 };

// Whether the down-projection runs in groups of four workgroups (kernels for r > 8 only): the
// rotation by half the grid has to keep groups together.
__device__ __forceinline__ bool down_grouped(const MegaArgs& a) { return (a.nwg & 7) == 0 && (a.wd.Nt & 3) == 0; }

// Phase number ph = 4 * layer + StreamPhase, or 4 * L for the vocabulary head.  The one place
// that says which matrix and which tile rotation a phase has: producers and consumers both ask
// here.  (Workgroups with one tile more than the others alternate between the halves of the
// grid from layer to layer.)
template <bool GROUPED>
__device__ __forceinline__ PhasePlan stream_phase(const MegaArgs& a, int ph, int wg, int wave) {
    const int nwg = a.nwg;
    if (ph >= 4 * a.L)
        return plan_phase(reinterpret_cast<const bf16x8*>(a.wbase + a.lm.off), a.lm.Nt, a.lm.Ks, wg, nwg, 0, wave);
    const int l = ph >> 2, k = ph & 3;
    const char* lb = a.wbase + a.layer0_off + size_t(l) * a.layer_stride;
    const int half = nwg / 2;
    if (k == SP_QKV)
        return plan_phase(reinterpret_cast<const bf16x8*>(lb + a.qkv.off), a.qkv.Nt, a.qkv.Ks, wg, nwg, (l & 1) * half, wave);
    if (k == SP_WO)
        return plan_phase(reinterpret_cast<const bf16x8*>(lb + a.wo.off), a.wo.Nt, a.wo.Ks, wg, nwg, (l & 1) * half, wave);
    if (k == SP_GU)
        return plan_phase(reinterpret_cast<const bf16x8*>(lb + a.gu.off), a.gu.Nt, a.gu.Ks, wg, nwg, 0, wave);
    if constexpr (GROUPED) {
        if (down_grouped(a))
            return plan_phase_grouped(reinterpret_cast<const bf16x8*>(lb + a.wd.off), a.wd.Nt, a.wd.Ks, wg, nwg,
                                      ((l + 1) & 1) * half, wave);
    }
    return plan_phase(reinterpret_cast<const bf16x8*>(lb + a.wd.off), a.wd.Nt, a.wd.Ks, wg, nwg, ((l + 1) & 1) * half, wave);
}

// ---- producer ----------------------------------------------------------------------------------
// Walks the stream of wavefront pair w: kRing loads in flight in a static register ring, each
// arrival written to the next FIFO slot (LDS addresses are dynamic, register indices are not).
// Waits only for FIFO space.  Once the step has failed (a bounded wait ran out somewhere) nobody
// waits any more: both sides run through their loops and the kernel ends.
//
// A wavefront issues an instruction every few cycles at best, a taken branch costs a pipeline
// refill, and a fragment is due every ~150 ns: the per-fragment path is a few dozen instructions
// without a taken branch (the next address is the last one + 1 KiB: stream order), everything
// else happens once per phase or when the FIFO is full.
//
// GROUPED (the kernels for r > 8): a phase planned by plan_phase_grouped interleaves four runs, one
// per tile of the batch.  The ring is unrolled, slot j always holds stream index n = j (mod 8), so
// the fragment with stream index n carries tile n & 3 (a fixed offset per ring slot: no counter,
// no select), and the k-step offset moves on behind the fourth fragment of a k-step, which is the
// slot with n & 3 == (rho + 3) & 3, rho = stream index of the phase's first fragment & 3.  The
// consumer, which has the same count, knows rho and which tile each of its accumulators holds.
// Plain phases are the same code with zero tile offsets and a step behind every fragment: one
// scalar addition more per fragment than the kernels for r <= 8 have.
template <bool GROUPED>
__device__ __forceinline__ void producer(const MegaArgs& a, MegaSmem& sm, int w, int lane, int wg) {
    const int n_ph = 4 * a.L + 1;
    int ph = -1;
    // the next load: resource, scalar offset, fragments left in the phase (0: the stream has ended)
    __amdgpu_buffer_rsrc_t cur_rs = make_rsrc(a.wbase, 0);
    uint32_t cur_off = 0, left = 0, issued = 0;
    uint32_t tile_off[4] = {0u, 0u, 0u, 0u}, step_behind[4] = {1024u, 1024u, 1024u, 1024u};
    uint32_t batches_left = 0u, per_batch = 0u, batch_base = 0u, batch_skip = 0u;
    auto next_phase = [&]() {
        if constexpr (GROUPED) {
            if (batches_left != 0u) {  // the next batch of a grouped phase
                --batches_left;
                batch_base += batch_skip;
                cur_off = batch_base;
                left = per_batch;
                return;
            }
        }
        while (++ph < n_ph) {
            const PhasePlan P = stream_phase<GROUPED>(a, ph, wg, w);
            left = uint32_t(P.cnt) * uint32_t(P.s1 - P.s0);
            if (left == 0) continue;
            cur_rs = make_rsrc(P.w, P.bytes);
            cur_off = P.first;
            if constexpr (GROUPED) {
                if (P.stride != 0u) {
                    const uint32_t last = (issued + 3u) & 3u;  // `issued` already counts the fragment before this phase
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        tile_off[u] = uint32_t(u) * P.stride;
                        step_behind[u] = uint32_t(u) == last ? 1024u : 0u;
                    }
                    per_batch = 4u * uint32_t(P.s1 - P.s0);
                    batches_left = left / per_batch - 1u;
                    left = per_batch;
                    batch_base = P.first;
                    batch_skip = P.batch_skip;
                } else {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        tile_off[u] = 0u;
                        step_behind[u] = 1024u;
                    }
                    batches_left = 0u;
                }
            }
            if (a.ts && w == 0 && lane == 0 && (ph >> 2) == a.ts_layer) a.ts[size_t(wg) * 32 + 17 + (ph & 3)] = wall_clock64();
            return;
        }
        left = 0;
        cur_off = 0;
        if constexpr (GROUPED) {
#pragma unroll
            for (int u = 0; u < 4; ++u) tile_off[u] = 0u;
        }
    };
    next_phase();
    uint32_t pushed = 0, head_seen = 0, pofs = 0;
    bool dead = false;
    // Every ring step is the same straight line on every path: wait for the slot's load, write it
    // to LDS (to a dump slot once the stream has ended), issue the slot's next load (an out-of-range
    // lane offset once the stream has ended: zeros, no memory access).  The scalar bookkeeping in
    // between may branch, the memory operations never do: the compiler's wait in front of a slot's
    // use then leaves exactly the other kRing - 1 loads in flight.
    auto issue = [&](bf16x8& dst, int slot) {
        const bool real = left != 0;
        int voff = real ? lane * 16 : kOutOfRange;
        uint32_t soff = cur_off;
        if constexpr (GROUPED) soff += tile_off[slot & 3];
        asm volatile("" : "+s"(soff), "+v"(voff));  // one load here, not one per incoming path
        dst = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(cur_rs, voff, int(soff), kAuxNT));
        if (real) {
            ++issued;
            if constexpr (GROUPED)
                cur_off += step_behind[slot & 3];
            else
                cur_off += 1024u;
            if (__builtin_expect(--left == 0, 0)) next_phase();
        }
    };
    auto push = [&](const bf16x8& v) {
        const bool real = pushed < issued;
        if (__builtin_expect(real && !dead && pushed - head_seen >= uint32_t(kFifo), 0)) {
            uint32_t spins = 0;
            while (true) {
                head_seen = lds_peek(&sm.head[w]);
                if (pushed - head_seen < uint32_t(kFifo)) break;
                __builtin_amdgcn_s_sleep(1);
                if (++spins > kLdsSpinLimit || (spins & 63u) == 0 && lds_peek(reinterpret_cast<uint32_t*>(&sm.failed)) != 0) {
                    dead = true;
                    lds_post(reinterpret_cast<uint32_t*>(&sm.failed), 1u);
                    break;
                }
            }
        }
        asm volatile("" ::: "memory");
        uint4v* dst = real ? reinterpret_cast<uint4v*>(reinterpret_cast<char*>(&sm.fifo[w][0][lane]) + pofs) : &sm.dump[lane];
        *dst = __builtin_bit_cast(uint4v, v);
        asm volatile("" ::: "memory");
        // LDS runs a wavefront's instructions in order: the count lands after the fragment
        pushed += real ? 1u : 0u;
        pofs = real ? (pofs + 1024u == uint32_t(kFifo) * 1024u ? 0u : pofs + 1024u) : pofs;
        lds_post(&sm.tail[w], pushed);
    };
    bf16x8 rg[kRing];
#pragma unroll
    for (int j = 0; j < kRing; ++j) issue(rg[j], j);
    while (pushed < issued) {
#pragma unroll
        for (int j = 0; j < kRing; ++j) {
            push(rg[j]);
            issue(rg[j], j);
        }
    }
}

// Consumer side of a FIFO (wavefront-uniform state).
struct FifoC {
    uint32_t head, tail_seen;  // in fragments
    uint32_t pos;              // slot of the next fragment
    bool dead;
    uint32_t waited;           // 100 MHz ticks spent waiting for fragments (read by the phase timeline)
};

// Wait until `need` fragments are there.
__device__ __forceinline__ void fifo_wait(MegaSmem& sm, FifoC& f, int w, uint32_t need) {
    if (__builtin_expect(f.tail_seen - f.head >= need, 1)) return;
    const unsigned long long w0 = wall_clock64();
    uint32_t spins = 0;
    while (!f.dead) {
        f.tail_seen = lds_peek(&sm.tail[w]);
        if (f.tail_seen - f.head >= need) break;
        __builtin_amdgcn_s_sleep(1);
        if (++spins > kLdsSpinLimit || (spins & 63u) == 0 && lds_peek(reinterpret_cast<uint32_t*>(&sm.failed)) != 0) {
            f.dead = true;
            lds_post(reinterpret_cast<uint32_t*>(&sm.failed), 1u);
        }
    }
    f.waited += uint32_t(wall_clock64() - w0);
    asm volatile("" ::: "memory");
}

// ---- sampling ------------------------------------------------------------------------------------
// Temperature > 0: the target's token for a position is a draw from softmax(logits / T), taken as
// arg-max of logits / T + G with G standard Gumbel noise (the maximum of Gumbel-perturbed logits is
// distributed as the softmax).  The noise is a pure function of (seed, position, token id): a
// counter-based generator, so a position gets the same draw whether its row is computed in a
// verification step or in a plain decode step, and verification reproduces token-by-token
// sampling exactly.  32-bit mixer: two-multiply xorshift finaliser ("lowbias32", C. Wellons,
// public domain); 24 bits of it give u = (k + 1/2) / 2^24 in (0, 1), exact in fp32.
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}
__device__ __forceinline__ uint32_t gumbel_row_key(uint32_t seed_lo, uint32_t seed_hi, uint32_t pos) {
    return mix32(mix32(mix32(seed_lo ^ 0x243f6a88u) ^ seed_hi) ^ pos);
}
__device__ __forceinline__ float gumbel_noise(uint32_t row_key, uint32_t token) {
    const uint32_t h = mix32(row_key + token * 0x9e3779b9u);
    const float u = (float(h >> 8) + 0.5f) * (1.0f / 16777216.0f);
    return -logf(-logf(u));
}

enum MegaEpi { ME_QKV = 0, ME_RESID = 1, ME_SWIGLU = 2, ME_LM = 3, ME_LM_TOPK = 4 };

// Running state of one thread across the batches of the vocabulary phase when the phase keeps a
// per-row top-k and a log-sum-exp (draft side) instead of the arg-max.
struct LmState {
    unsigned long long run[2];  // this lane's share of its row's sixteen best keys so far
    float m, s;                 // running maximum and sum of exp(value - m) over this lane's columns
};

struct EpiArgs {
    int32_t layer;
    int32_t ts0;  // timeline slots of this phase: ts0 first activations in, ts0+1 k-loop left, ts0+2 ticks spent waiting for fragments (not for the down-projection, whose third slot would be attention's); <= 0: none
    const float* ss_in;      // [32 rows][d/16] partial sums of squares of the input rows (norm phases)
    // RESID
    const float* xres_old;
    float* xres_new;
    __bf16* xfrag_new;
    float* ss_new;
    const float* gain_next;
    // QKV
    __bf16* qfrag;
    __bf16* kpool;
    __bf16* vpool;
    // SWIGLU
    __bf16* actfrag;
    // LM with top-k
    LmState* lm;
};

struct NoHook {
    __device__ __forceinline__ void operator()() const {}
};

// ---- one GEMM phase, consumer side ---------------------------------------------------------------
// out[m][n] = sum_k x[m][k] W[n][k] for this workgroup's n-tiles; the four wavefronts cut K.
// Fragments are popped GROUP at a time (SG k-steps x NB tiles); the activations (B operand) sit
// in a register ring of XD k-steps, each slot refilled right after its use with the step XD
// further on, so their latency hides behind a whole ring cycle.  `after_k` runs once, after the
// last k-loop of the phase and before its reduction and epilogue.
//
// PK ("packed halves", r <= 8): the 16 activation columns of the matrix instruction hold the high
// halves of the (at most eight) rows in columns 0-7 and their low halves in columns 8-15, so one
// instruction per weight fragment does what otherwise takes two, one operand load per k-step
// fetches the whole contiguous rp*128-byte run, and the two partial products of a row meet in the
// reduction.  (The ring stays eight k-steps deep: sixteen measured 3 % slower.)
//
// GRP4 (r > 8, residual epilogue): the phase was planned by plan_phase_grouped.  The batch's four
// tiles belong to the four positions of the group (tile ids t_first + i, the next batch nwg
// further on); what the workgroup has after its own reduction is the sum over ITS quarter of K,
// so the four workgroups hand their blocks over in memory and the last one to arrive adds the four
// (always in the order of the quarters, whoever comes last) and runs the epilogue for all four
// tiles.
template <int NB, int MT, int EPI, bool PK, typename Hook = NoHook, bool GRP4 = false>
__device__ __forceinline__ void gemm_phase(const MegaArgs& a, const PhasePlan& P, const __bf16* xf, uint32_t xf_bytes,
                                           const EpiArgs& ea, FifoC& fc, MegaSmem& sm, int wave, int lane,
                                           uint32_t& cgen, Hook after_k = Hook()) {
    // fragments per pop: eight; outside the packed-halves mode every k-step holds two (r <= 16) or
    // four (r <= 32) activation operands, and smaller groups and rings leave the registers for
    // them: four fragments in narrow batches at r <= 16 (8B shape, r = 16: 3.68 -> 3.59 ms), one
    // k-step of the batch (at least two fragments) at r <= 32 (r = 32: 4.81 -> 4.39 ms)
    constexpr int GRP = PK ? kGroup : (MT == 2 ? (NB < 2 ? 2 : NB) : (NB < kGroup ? kGroup / 2 : kGroup));
    static_assert(NB <= GRP && GRP % NB == 0, "batch width");
    constexpr int SG = GRP / NB;  // k-steps per group
    // k-steps in the activation ring (a multiple of SG): eight single-operand steps, four
    // two-operand steps, two four-operand steps
    static_assert(!PK || MT == 1, "packed halves: one row tile");
    static_assert(!GRP4 || (!PK && NB == 4 && EPI == ME_RESID), "grouped phases: four tiles, residual epilogue");
    const int t_inner = GRP4 ? 1 : a.nwg, t_batch = GRP4 ? a.nwg : NB * a.nwg;  // tile id steps inside a batch, between batches
    // grouped phases: the fragment with stream index n carries tile n & 3, so accumulator i of this
    // wavefront holds tile (i + rho) & 3, rho = stream index of the phase's first fragment & 3
    const uint32_t rho = GRP4 ? (fc.head & 3u) : 0u;
    constexpr int XD = PK ? 8 : (MT == 2 ? 2 : 4);
    static_assert(XD % SG == 0, "ring of whole groups");
    constexpr int COLS = 16 * MT;
    constexpr int NSUB = NB * MT > 8 ? 2 : 1, NBS = NB / NSUB;  // reduction rounds per batch, tiles per round
    const int tid = opaque_v(threadIdx.x);
    lane = tid & 63;
    const int r = a.r, rp = a.rp;

    const __amdgpu_buffer_rsrc_t xr = make_rsrc(xf, xf_bytes);
    int xoff[MT];
#pragma unroll
    for (int j = 0; j < MT; ++j) {
        if constexpr (PK) {
            const int row = lane & 7, half = (lane >> 3) & 1;
            xoff[j] = row < r ? ((lane >> 4) * rp + row) * 32 + half * 16 : kOutOfRange;
        } else {
            const int row = j * 16 + (lane & 15);
            xoff[j] = row < r ? ((lane >> 4) * rp + row) * 32 : kOutOfRange;
        }
    }
    const int n_batches = (P.cnt + NB - 1) / NB;
    const int n_steps = P.s1 - P.s0;
    const int n_xb = (n_steps + XD - 1) / XD;
    const int vtot = n_xb * XD;  // virtual k-steps of one batch (the tail beyond s1 reads zeros)

    bf16x8 xh[XD][MT], xl[XD][MT];
    // Activations of k-steps past the wavefront's share are whatever the buffer holds there (zeros
    // past its end): the weight fragments of such steps are zero, so they add nothing.
    const uint32_t xstep = uint32_t(rp) * 128u;
    auto load_x = [&](uint32_t soff, bf16x8 (&h)[MT], bf16x8 (&l)[MT]) {
#pragma unroll
        for (int j = 0; j < MT; ++j) {
            h[j] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(xr, xoff[j], int(soff), 0));
            if constexpr (!PK)
                l[j] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(xr, xoff[j] + 16, int(soff), 0));
        }
    };
    const uint32_t xs0 = uint32_t(P.s0) * xstep;
    uint32_t xs_next = xs0;  // offset of the next k-step to fetch, vn_next its (virtual) index in the batch
    int vn_next = 0;
    auto refill = [&](bf16x8 (&h)[MT], bf16x8 (&l)[MT]) {
        load_x(xs_next, h, l);
        xs_next += xstep;
        if (++vn_next == vtot) {  // every batch uses the same activations
            vn_next = 0;
            xs_next = xs0;
        }
    };
    if (n_batches > 0 && n_xb > 0) {
#pragma unroll
        for (int u = 0; u < XD; ++u) refill(xh[u], xl[u]);
    }
    // Loads whose results are only needed after the k-loop are issued now, behind the first
    // activations (loads return in issue order): the per-tile sums of squares behind the RMSNorm
    // scale (SSL lanes per row, SSQ groups of four tiles each) ...
    constexpr int SSL = kMegaThreads / kMaxR, SSQ = 8;
    float4 ssv[SSQ];
    const int ss_row = tid / SSL, ss_sub = tid % SSL, n_part = a.d >> 4, n_grp = n_part >> 2;
    if constexpr (EPI != ME_RESID) {
#pragma unroll
        for (int q = 0; q < SSQ; ++q) {
            const int g = ss_sub + SSL * q;
            ssv[q] = (ss_row < r && g < n_grp) ? *reinterpret_cast<const float4*>(ea.ss_in + size_t(ss_row) * n_part + 4 * g)
                                               : float4{0.f, 0.f, 0.f, 0.f};
        }
    }
    // ... and the old residual values and next gains of the tile this thread will finish
    float xo8[8], gn8[8];
    if constexpr (EPI == ME_RESID) {
        const int c = tid & 1, m = (tid >> 1) % kMaxR, i = tid / (2 * kMaxR);
        const bool on = i < min(NB, P.cnt) && m < r;
#pragma unroll
        for (int e = 0; e < 8; ++e) xo8[e] = gn8[e] = 0.f;
        if (on) {
            const int n0 = (P.t_first + i * t_inner) * 16 + c * 8;
            const float4 x0 = *reinterpret_cast<const float4*>(ea.xres_old + size_t(m) * a.d + n0);
            const float4 x1 = *reinterpret_cast<const float4*>(ea.xres_old + size_t(m) * a.d + n0 + 4);
            const float4 g0 = *reinterpret_cast<const float4*>(ea.gain_next + n0);
            const float4 g1 = *reinterpret_cast<const float4*>(ea.gain_next + n0 + 4);
            xo8[0] = x0.x; xo8[1] = x0.y; xo8[2] = x0.z; xo8[3] = x0.w;
            xo8[4] = x1.x; xo8[5] = x1.y; xo8[6] = x1.z; xo8[7] = x1.w;
            gn8[0] = g0.x; gn8[1] = g0.y; gn8[2] = g0.z; gn8[3] = g0.w;
            gn8[4] = g1.x; gn8[5] = g1.y; gn8[6] = g1.z; gn8[7] = g1.w;
        }
    }

    bool hook_done = false;
    const uint32_t waited0 = fc.waited;
    const bool gts = a.ts && ea.ts0 > 0 && ea.layer == a.ts_layer && tid == 0;
    if (gts) {
        asm volatile("" ::"v"(xh[0][0]));  // the first activations have arrived
        a.ts[size_t(blockIdx.x) * 32 + ea.ts0] = wall_clock64();
    }

    for (int b = 0; b < n_batches; ++b) {
        floatx4 acc[NB][MT];
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int j = 0; j < MT; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
        const int nvalid = min(NB, P.cnt - b * NB);

        for (int xb = 0; xb < n_xb; ++xb) {
#pragma unroll
            for (int gg = 0; gg < XD / SG; ++gg) {
                const int st0 = xb * XD + gg * SG;  // first (virtual) k-step of the group
                int nvs = n_steps - st0;
                nvs = nvs > SG ? SG : nvs;
                if (nvs > 0) {
                    // the group: nvs k-steps x nvalid tiles, step-major, in consecutive FIFO slots
                    const uint32_t need = uint32_t(nvs * nvalid);
                    fifo_wait(sm, fc, wave, need);
                    bf16x8 fr[SG][NB];
                    const bool straight = fc.pos + uint32_t(GRP) <= uint32_t(kFifo);  // no wrap inside the group
                    if (straight && nvs == SG && (SG == 1 || nvalid == NB)) {
                        // Static slot offsets.  With one k-step per group the slots of tiles the batch
                        // does not have hold stale bits: they only reach those tiles' accumulators,
                        // which nobody reads.
                        const uint4v* grp = &sm.fifo[wave][fc.pos][lane];
#pragma unroll
                        for (int k = 0; k < GRP; ++k) fr[k / NB][k % NB] = __builtin_bit_cast(bf16x8, grp[k * 64]);
                    } else {
#pragma unroll
                        for (int u = 0; u < SG; ++u)
#pragma unroll
                            for (int i = 0; i < NB; ++i) {
                                fr[u][i] = __builtin_bit_cast(bf16x8, uint4v{0u, 0u, 0u, 0u});
                                if (u < nvs && i < nvalid) {
                                    uint32_t sl = fc.pos + uint32_t(u * nvalid + i);
                                    sl = sl >= uint32_t(kFifo) ? sl - uint32_t(kFifo) : sl;
                                    fr[u][i] = __builtin_bit_cast(bf16x8, sm.fifo[wave][sl][lane]);
                                }
                            }
                    }
                    // LDS runs a wavefront's instructions in order: the slots are read before this lands
                    asm volatile("" ::: "memory");
                    fc.head += need;
                    fc.pos += need;
                    fc.pos = fc.pos >= uint32_t(kFifo) ? fc.pos - uint32_t(kFifo) : fc.pos;
                    lds_post(&sm.head[wave], fc.head);
#pragma unroll
                    for (int u = 0; u < SG; ++u) {
                        const int slot = gg * SG + u;
#pragma unroll
                        for (int i = 0; i < NB; ++i)
#pragma unroll
                            for (int j = 0; j < MT; ++j) {
                                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fr[u][i], xh[slot][j], acc[i][j], 0, 0, 0);
                                if constexpr (!PK)
                                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fr[u][i], xl[slot][j], acc[i][j], 0, 0, 0);
                            }
                    }
                }
#pragma unroll
                for (int u = 0; u < SG; ++u) refill(xh[gg * SG + u], xl[gg * SG + u]);
            }
        }
        if (b + 1 == n_batches) {
            if (gts) {
                a.ts[size_t(blockIdx.x) * 32 + ea.ts0 + 1] = wall_clock64();
                if (ea.ts0 + 2 < 29) a.ts[size_t(blockIdx.x) * 32 + ea.ts0 + 2] = fc.waited - waited0;  // (29.. belong to attention)
            }
            after_k();
            hook_done = true;
        }
        if constexpr (EPI != ME_RESID) {
            if (b == 0) {
                float sq = 0.f;
#pragma unroll
                for (int q = 0; q < SSQ; ++q) sq += (ssv[q].x + ssv[q].y) + (ssv[q].z + ssv[q].w);
                if (ss_row < r)
                    for (int g = ss_sub + SSL * SSQ; g < n_grp; g += SSL) {
                        const float4 v = *reinterpret_cast<const float4*>(ea.ss_in + size_t(ss_row) * n_part + 4 * g);
                        sq += (v.x + v.y) + (v.z + v.w);
                    }
#pragma unroll
                for (int o = 1; o < SSL; o <<= 1) sq += __shfl_xor(sq, o);
                if (ss_sub == 0 && ss_row < r) sm.row_scale[ss_row] = 1.0f / sqrtf(sq * a.inv_d + a.eps);
            }
        }

        // Reduction and epilogue run on at most eight tile x row-tile blocks at a time (the LDS
        // staging is sized for that): wide batches with two row tiles take two rounds.
#pragma unroll
        for (int sb = 0; sb < NSUB; ++sb) {
        const int nvalid_s = max(0, min(NBS, nvalid - sb * NBS));
        // ---- reduce the four wavefronts (fixed order) --------------------------------------
#pragma unroll
        for (int i = 0; i < NBS; ++i)
#pragma unroll
            for (int j = 0; j < MT; ++j)
                *reinterpret_cast<floatx4*>(&sm.red[(wave * NBS * MT + (GRP4 ? int((uint32_t(i) + rho) & 3u) : i) * MT + j) * 256 +
                                                    lane * 4]) = acc[sb * NBS + i][j];
        cbar(sm, cgen);
        for (int e = tid; e < NBS * MT * 256; e += kMegaThreads) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < kMegaWaves; ++w) s += sm.red[w * NBS * MT * 256 + e];
            const int t = e >> 8, l = (e & 255) >> 2, v = e & 3;
            const int i = t / MT, j = t % MT;
            if constexpr (PK) {
                // column c < 8 carries the high halves' product of row c, column c + 8 the low halves'
                if ((l & 15) >= 8) continue;
#pragma unroll
                for (int w = 0; w < kMegaWaves; ++w) s += sm.red[w * NBS * MT * 256 + e + 32];
            }
            sm.tile[(i * 16 + (l >> 4) * 4 + v) * COLS + j * 16 + (l & 15)] = s;
        }
        cbar(sm, cgen);

        // ---- epilogue ----------------------------------------------------------------------------
        const int tile0 = P.t_first + b * t_batch + sb * NBS * t_inner;  // tile i of the sub-batch: tile0 + i * t_inner
        bool finish = true;
        if constexpr (GRP4) {
            // this workgroup's block (its quarter of K, the batch's four tiles) goes to memory ...
            constexpr int BLK = 4 * 16 * kMaxR;  // floats per (group of four tiles, quarter)
            constexpr int NEL = NB * 16 * COLS;  // of which this kernel uses
            float* grp = a.dpart + size_t(tile0 >> 2) * (4 * BLK);
            const int e0 = tid * 8;
            if (e0 < NEL) {
                float v8[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) v8[q] = sm.tile[e0 + q];
                st_dev_f32x8(grp + P.quarter * BLK, e0, v8);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0);
            cbar(sm, cgen);
            int* flag = reinterpret_cast<int*>(&sm.wgt[(kMegaWaves + 2) * 16]);
            if (tid == 0) {
                const uint32_t prev = __hip_atomic_fetch_add(&a.dcount[tile0 >> 2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                *flag = prev == 3u;
            }
            cbar(sm, cgen);
            finish = *flag != 0;
            if (finish) {
                // ... and the last of the four adds them up, quarter by quarter
                const __amdgpu_buffer_rsrc_t prs = make_rsrc(grp, 4 * BLK * 4);
                if (e0 < NEL) {
                    uint4v lo4[4], hi4[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        lo4[q] = __builtin_amdgcn_raw_buffer_load_b128(prs, e0 * 4, q * BLK * 4, kAuxDev);
                        hi4[q] = __builtin_amdgcn_raw_buffer_load_b128(prs, e0 * 4 + 16, q * BLK * 4, kAuxDev);
                    }
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float s0 = 0.f, s1 = 0.f;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            s0 += __uint_as_float(lo4[q][v]);
                            s1 += __uint_as_float(hi4[q][v]);
                        }
                        sm.tile[e0 + v] = s0;
                        sm.tile[e0 + 4 + v] = s1;
                    }
                }
                if (tid == 0) __hip_atomic_store(&a.dcount[tile0 >> 2], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                cbar(sm, cgen);
            }
        }
        if constexpr (EPI == ME_RESID) {
            // work item: (tile i, row m, half c of the 16 columns); lanes 2q and 2q+1 share a row
            const int c = tid & 1, m = (tid >> 1) % kMaxR, i = tid / (2 * kMaxR);
            const bool on = i < nvalid_s && m < r && finish;
            float ssum = 0.f;
            if (on) {
                const int n0 = (tile0 + i * t_inner) * 16 + c * 8;
                if (b > 0) {  // later batches were not pre-loaded
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        xo8[e] = ea.xres_old[size_t(m) * a.d + n0 + e];
                        gn8[e] = ea.gain_next[n0 + e];
                    }
                }
                float nv[8], gv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    nv[e] = xo8[e] + sm.tile[(i * 16 + c * 8 + e) * COLS + m];
                    ssum += nv[e] * nv[e];
                    gv[e] = nv[e] * gn8[e];
                }
                st_dev_f32x8(ea.xres_new, uint32_t(m) * a.d + n0, nv);
                st_dev_frag8(ea.xfrag_new, frag_index(n0, m, rp), gv);
            }
            ssum += __shfl_xor(ssum, 1);
            if (on && c == 0) st_agent(ea.ss_new + size_t(m) * (a.d >> 4) + (tile0 + i * t_inner), ssum);
            static_assert(NBS * 2 * kMaxR <= kMegaThreads, "one pass");
        } else if constexpr (EPI == ME_SWIGLU) {
            const int m = tid % kMaxR, i = tid / kMaxR;
            if (i < nvalid_s && m < r) {
                const float sc = sm.row_scale[m];
                float av[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float g = sm.tile[(i * 16 + e) * COLS + m] * sc;
                    const float u = sm.tile[(i * 16 + 8 + e) * COLS + m] * sc;
                    // SiLU with the hardware exp2 and reciprocal (1 ulp each; the result is rounded to
                    // bf16 high + low halves afterwards)
                    av[e] = g * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g)) * u;
                }
                const int f0 = (tile0 + i * a.nwg) * 8;
                st_dev_frag8(ea.actfrag, frag_index(f0, m, rp), av);
            }
        } else if constexpr (EPI == ME_LM || EPI == ME_LM_TOPK) {
            if (a.logits) {
                for (int e = tid; e < NBS * 16 * r; e += kMegaThreads) {
                    const int nl = e % (NBS * 16), m = e / (NBS * 16);
                    const int i = nl >> 4;
                    const int n = (tile0 + i * a.nwg) * 16 + (nl & 15);
                    if (i < nvalid_s && n < a.V) a.logits[size_t(m) * a.V + n] = sm.tile[nl * COLS + m] * sm.row_scale[m];
                }
            }
            if constexpr (EPI == ME_LM_TOPK) {
                // Draft side (Cache Construction, eqs. (1)-(2)): per row the k most probable tokens and
                // the log-sum-exp that turns their logits into probabilities, without storing the
                // row.  The lanes of a row are consecutive (16 of them with one row tile, 8 with
                // two), each owns eight columns of the batch and a share of the row's running best
                // sixteen; sixteen rounds of "largest key among the row's lanes" rebuild that list
                // from the old list and the new columns.  Keys are (ordered logit, ~token): unique,
                // so the lane that holds a round's winner knows it and drops it.
                constexpr int LPR = kMegaThreads / COLS, CPL = NBS * 16 / LPR, RUN = 16 / LPR;
                static_assert(CPL == 8 && RUN * LPR == 16, "eight columns per lane, sixteen entries per row");
                LmState& lm = *ea.lm;
                const int m = tid / LPR, p = tid % LPR;
                const float sc = m < r ? sm.row_scale[m] : 0.f;
                unsigned long long cand[CPL];
#pragma unroll
                for (int q = 0; q < CPL; ++q) {
                    const int nl = p * CPL + q, i = nl >> 4;
                    const int n = (tile0 + i * a.nwg) * 16 + (nl & 15);
                    cand[q] = 0ull;
                    if (m < r && i < nvalid_s && n < a.V) {
                        const float val = sm.tile[nl * COLS + m] * sc;
                        cand[q] = (static_cast<unsigned long long>(float_key(val)) << 32) | (0xffffffffu - uint32_t(n));
                        if (val > lm.m) {
                            lm.s = lm.s * __expf(lm.m - val) + 1.f;
                            lm.m = val;
                        } else {
                            lm.s += __expf(val - lm.m);
                        }
                    }
                }
                unsigned long long nr[RUN];
#pragma unroll
                for (int u = 0; u < RUN; ++u) nr[u] = 0ull;
#pragma unroll 1
                for (int j = 0; j < 16; ++j) {
                    unsigned long long loc = 0ull;
#pragma unroll
                    for (int q = 0; q < CPL; ++q) loc = cand[q] > loc ? cand[q] : loc;
#pragma unroll
                    for (int u = 0; u < RUN; ++u) loc = lm.run[u] > loc ? lm.run[u] : loc;
                    unsigned long long best = loc;
#pragma unroll
                    for (int o = 1; o < LPR; o <<= 1) {
                        const unsigned long long other = __shfl_xor(best, o);
                        best = other > best ? other : best;
                    }
                    if (best != 0ull) {
#pragma unroll
                        for (int q = 0; q < CPL; ++q) cand[q] = cand[q] == best ? 0ull : cand[q];
#pragma unroll
                        for (int u = 0; u < RUN; ++u) lm.run[u] = lm.run[u] == best ? 0ull : lm.run[u];
                    }
                    if (p == j % LPR) {
#pragma unroll
                        for (int u = 0; u < RUN; ++u) nr[u] = (j / LPR == u) ? best : nr[u];
                    }
                }
#pragma unroll
                for (int u = 0; u < RUN; ++u) lm.run[u] = nr[u];
            }
            constexpr int PARTS = kMegaThreads / COLS;
            constexpr int ROWS_PER = NBS * 16 / PARTS;
            static_assert(ROWS_PER >= 1, "rows per thread");
            {
                const int m = tid % COLS, part = tid / COLS;
                unsigned long long best = 0ull;
                if (m < r) {
                    const float sc = sm.row_scale[m];
                    // row m predicts the token at position ctx_len + m + 1
                    const uint32_t rkey = gumbel_row_key(a.seed_lo, a.seed_hi, uint32_t(a.ctx_len + m + 1));
#pragma unroll
                    for (int q = 0; q < ROWS_PER; ++q) {
                        const int nl = part * ROWS_PER + q, i = nl >> 4;
                        const int n = (tile0 + i * a.nwg) * 16 + (nl & 15);
                        if (i < nvalid_s && n < a.V) {
                            float val = sm.tile[nl * COLS + m] * sc;
                            if (a.inv_temp > 0.f) val = val * a.inv_temp + gumbel_noise(rkey, uint32_t(n));
                            const unsigned long long key =
                                (static_cast<unsigned long long>(float_key(val)) << 32) |
                                (0xffffffffu - uint32_t(n));
                            best = key > best ? key : best;
                        }
                    }
                }
                sm.part_best[part * COLS + m] = best;
            }
            cbar(sm, cgen);
            if (tid < r) {
                unsigned long long best = sm.wg_best[tid];
                for (int part = 0; part < PARTS; ++part) {
                    const unsigned long long k = sm.part_best[part * COLS + tid];
                    best = k > best ? k : best;
                }
                sm.wg_best[tid] = best;
            }
        } else {  // ME_QKV
            // packed rows: [q heads | k heads | v heads]; in q and k heads row 2p is element p of the
            // head and row 2p+1 its rotation partner p + h/2.  Work item: (tile, row m, which half).
            const int which = tid & 1, m = (tid >> 1) % kMaxR, i = tid / (2 * kMaxR);
            if (i < nvalid_s && m < r) {
                const int h = a.h, half = h >> 1;
                const int prow = (tile0 + i * a.nwg) * 16;
                const float sc = sm.row_scale[m];
                const int slot = a.slot0 + m;
                const int page = a.block_table[slot >> 4], tk = slot & 15;
                if (prow < a.qd + a.kvd) {
                    const bool is_q = prow < a.qd;
                    const int rel = is_q ? prow : prow - a.qd;
                    const int head = rel / h, p0 = (rel % h) >> 1;  // eight pairs p0 .. p0+7 (p0 % 8 == 0)
                    float ov[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float z0 = sm.tile[(i * 16 + 2 * e) * COLS + m] * sc;
                        const float z1 = sm.tile[(i * 16 + 2 * e + 1) * COLS + m] * sc;
                        const float cs = a.rope[m * half + p0 + e], sn = a.rope[kMaxR * half + m * half + p0 + e];
                        ov[e] = which == 0 ? z0 * cs - z1 * sn : z1 * cs + z0 * sn;
                    }
                    const int j0 = p0 + which * half;  // first of eight consecutive head elements
                    if (is_q) {
                        const int kvh = head / a.G, gl = head % a.G;
                        const int rho = m * a.G + gl;
#pragma unroll
                        for (int e = 0; e < 8; ++e) ov[e] *= a.inv_sqrt_h;
                        st_dev_frag8(ea.qfrag, ((size_t(kvh) * (a.G * kMaxR) + rho) * (h >> 3) + (j0 >> 3)) * 16, ov);
                    } else {
                        const size_t ko = (size_t(page) * a.Hkv + head) * (16 * h) + ((j0 >> 3) * 16 + tk) * 8;
                        uint4v w;
#pragma unroll
                        for (int e = 0; e < 8; e += 2)
                            w[e / 2] = pack_bf16(static_cast<__bf16>(ov[e]), static_cast<__bf16>(ov[e + 1]));
                        st_dev_b128(ea.kpool, uint32_t(ko * 2), w);
                    }
                }
            }
            // V rows: work item (tile, head element j of the tile); the r tokens of one element are
            // consecutive 2-byte slots inside a page row, written as the widest aligned stores
            const int jj = (tid & 1) * 8 + ((tid >> 1) & 7);
            const bool v_lane = ((tid >> 1) % kMaxR) < 8;
            if (i < nvalid_s && v_lane && (tile0 + i * a.nwg) * 16 >= a.qd + a.kvd) {
                const int h = a.h;
                const int rel = (tile0 + i * a.nwg) * 16 - a.qd - a.kvd + jj;
                const int head = rel / h, jg = rel % h;
                int m2 = 0;
                while (m2 < r) {
                    const int slot = a.slot0 + m2;
                    const int page = a.block_table[slot >> 4], tk = slot & 15;
                    const int run = min(r - m2, 16 - tk);
                    const size_t vb = (size_t(page) * a.Hkv + head) * (16 * h);
                    auto val = [&](int t) {
                        return static_cast<__bf16>(sm.tile[(i * 16 + jj) * COLS + m2 + t] * sm.row_scale[m2 + t]);
                    };
                    int q = 0;
                    while (q < run) {  // four consecutive aligned tokens are 8 contiguous bytes
                        const int t = tk + q;
                        __bf16* dst = ea.vpool + vb + v_page_index(jg, t);
                        if ((t & 3) == 0 && q + 4 <= run) {
                            const unsigned long long w = uint64_t(pack_bf16(val(q), val(q + 1))) |
                                                         (uint64_t(pack_bf16(val(q + 2), val(q + 3))) << 32);
                            __hip_atomic_store(reinterpret_cast<unsigned long long*>(dst), w, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                            q += 4;
                        } else if ((t & 1) == 0 && q + 2 <= run) {
                            __hip_atomic_store(reinterpret_cast<uint32_t*>(dst), pack_bf16(val(q), val(q + 1)),
                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            q += 2;
                        } else {
                            st_dev_bf16(dst, val(q));
                            q += 1;
                        }
                    }
                    // a page is opened by the call that writes its first slot: clear the slots behind
                    // the ones written, so that a later step never multiplies a zero probability with
                    // bits nobody stored (0 x NaN)
                    if (tk == 0) {
                        int t = run;
                        while (t < 16) {
                            __bf16* dst = ea.vpool + vb + v_page_index(jg, t);
                            if ((t & 3) == 0) {
                                __hip_atomic_store(reinterpret_cast<unsigned long long*>(dst), 0ull, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
                                t += 4;
                            } else if ((t & 1) == 0) {
                                __hip_atomic_store(reinterpret_cast<uint32_t*>(dst), 0u, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
                                t += 2;
                            } else {
                                st_dev_bf16(dst, static_cast<__bf16>(0.f));
                                t += 1;
                            }
                        }
                    }
                    m2 += run;
                }
            }
        }
        cbar(sm, cgen);  // red / tile are reused by the next batch
        }
    }
    if (!hook_done) after_k();
}

// ---- chain attention phase ------------------------------------------------------------------------
// Rows = the G query heads sharing one KV head x the r candidates; row (m, g) sees keys at
// positions <= ctx_len + m (the target verifies a plain chain, never a tree: Cache Correction,
// last paragraph).  Task = (kv head, 16-row tile, cut of the page list); the four consumer wavefronts of
// a workgroup take pages round-robin.  Per 16-token page: S^T = K Q^T on the matrix pipe (K page
// stored in operand order), online softmax per row with wavefront-level reductions,
// O^T += V^T P^T with the probability tile fed straight from the accumulator registers.
// Wavefront partials (max, sum, O) meet in LDS; cuts meet in global partials merged by whichever
// workgroup arrives last.  Pages that hold only old context do not depend on this step's QKV
// phase, so their loads are issued BEFORE the grid barrier that precedes attention.
struct AttnTask {
    int kvh, rt, split, pg0, pg1;
};

__device__ __forceinline__ AttnTask attn_task(const MegaArgs& a, int task) {
    AttnTask t;
    t.split = task % a.a_splits;
    t.rt = (task / a.a_splits) % a.row_tiles;
    t.kvh = task / (a.a_splits * a.row_tiles);
    t.pg0 = t.split * a.pages_per_split;
    t.pg1 = min(a.pages_used, t.pg0 + a.pages_per_split);
    return t;
}

template <int H>
__device__ __forceinline__ void attn_load_k(const MegaArgs& a, const __bf16* kpool, int kvh, int pid, int lane,
                                            bf16x8 (&kf)[H / 32]) {
    const size_t base = (size_t(pid) * a.Hkv + kvh) * (16 * H);
    const bf16x8* kp = reinterpret_cast<const bf16x8*>(kpool + base) + lane;
#pragma unroll
    for (int st = 0; st < H / 32; ++st) kf[st] = kp[st * 64];
}
template <int H>
__device__ __forceinline__ void attn_load_v(const MegaArgs& a, const __bf16* vpool, int kvh, int pid, int lane,
                                            short4v (&vf)[H / 16]) {
    const size_t base = (size_t(pid) * a.Hkv + kvh) * (16 * H);
    const uint4v* vp = reinterpret_cast<const uint4v*>(vpool + base) + lane;
#pragma unroll
    for (int i = 0; i < H / 32; ++i) {  // one 16-byte load = the operands of two 16-row tiles
        const uint4v w = vp[i * 64];
        vf[2 * i] = __builtin_bit_cast(short4v, uint2v{w[0], w[1]});
        vf[2 * i + 1] = __builtin_bit_cast(short4v, uint2v{w[2], w[3]});
    }
}
template <int H>
__device__ __forceinline__ void attn_load_page(const MegaArgs& a, const __bf16* kpool, const __bf16* vpool, int kvh,
                                               int pid, int lane, bf16x8 (&kf)[H / 32], short4v (&vf)[H / 16]) {
    attn_load_k<H>(a, kpool, kvh, pid, lane, kf);
    attn_load_v<H>(a, vpool, kvh, pid, lane, vf);
}

// Second half of an attention task: merge the four consumer wavefronts' partials in LDS, then
// either finish (context not cut) or hand the cut's partial over and let the last workgroup of
// this (kv head, row tile) merge all cuts.
template <int H>
__device__ __forceinline__ void attn_finish(MegaSmem& sm, float* apart, uint32_t* acount, __bf16* attfrag_l,
                                            int G, int rp, int R, int a_splits, int row_tiles, int task, int split,
                                            int kvh, int rt, uint32_t& cgen, unsigned long long* tsp) {
    constexpr int PART = 16 * (H + 2);
    const int tid = threadIdx.x;
        if (tid < 16) {
            float mg = -1e30f;
            for (int w = 0; w < kMegaWaves; ++w) mg = fmaxf(mg, sm.attn[w * PART + tid]);
            float l = 0.f;
            for (int w = 0; w < kMegaWaves; ++w) {
                const float f = __builtin_amdgcn_exp2f(sm.attn[w * PART + tid] - mg);
                sm.wgt[w * 16 + tid] = f;
                l += f * sm.attn[w * PART + 16 + tid];
            }
            sm.wgt[kMegaWaves * 16 + tid] = mg;
            sm.wgt[(kMegaWaves + 1) * 16 + tid] = l;
        }
        cbar(sm, cgen);
        // work item: (row, chunk of 8 head elements); H/8 * 16 <= 256 items
        const int row = tid / (H / 8), ch = tid % (H / 8);
        const bool item = tid < 16 * (H / 8);
        const int rr = rt * 16 + row;
        float v8[8];
        if (item) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                float acc = 0.f;
                for (int w = 0; w < kMegaWaves; ++w) acc += sm.wgt[w * 16 + row] * sm.attn[w * PART + 32 + row * H + ch * 8 + q];
                v8[q] = acc;
            }
        }
        float* att_part = apart + size_t(task) * PART;
        bool finish = a_splits == 1;
        float inv_l = 0.f;
        if (a_splits == 1) {
            if (item) inv_l = 1.0f / sm.wgt[(kMegaWaves + 1) * 16 + row];
        } else {
            // hand the cut's partial over; the last workgroup of this (kv head, row tile) merges
            if (item) st_dev_f32x8(att_part, 32 + row * H + ch * 8, v8);
            if (tid < 16) {
                st_agent(att_part + tid, sm.wgt[kMegaWaves * 16 + tid]);
                st_agent(att_part + 16 + tid, sm.wgt[(kMegaWaves + 1) * 16 + tid]);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0);
            cbar(sm, cgen);
            if (tsp && tid == 0) tsp[29] = wall_clock64();
            int* flag = reinterpret_cast<int*>(&sm.wgt[(kMegaWaves + 2) * 16]);
            if (tid == 0) {
                const uint32_t prev = __hip_atomic_fetch_add(&acount[kvh * row_tiles + rt], 1u, __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_AGENT);
                *flag = prev == uint32_t(a_splits) - 1;
            }
            cbar(sm, cgen);
            finish = *flag != 0;
            if (tsp && tid == 0) tsp[30] = wall_clock64();
            if (finish) {
                // One round trip per ten cuts: every work item fetches its row's (max, sum) pairs
                // and its own eight output values of those cuts together, then folds them in with a
                // running maximum.
                const int S = a_splits;
                const float* base = apart + size_t(task - split) * PART;
                const __amdgpu_buffer_rsrc_t prs = make_rsrc(base, uint32_t(S) * PART * 4);
                float mg = -1e30f, lg = 0.f;
#pragma unroll
                for (int q = 0; q < 8; ++q) v8[q] = 0.f;
                constexpr int CH = 10;
                for (int s0 = 0; s0 < S; s0 += CH) {
                    uint32_t mw[CH], lw[CH];
                    uint4v p0[CH], p1[CH];
#pragma unroll
                    for (int c = 0; c < CH; ++c) {
                        // cuts past the last one: an offset beyond the buffer, the loads return zeros
                        const uint32_t cut = uint32_t(s0 + c) * PART * 4;
                        const int lane_off = (item && s0 + c < S) ? 0 : kOutOfRange;
                        mw[c] = __builtin_amdgcn_raw_buffer_load_b32(prs, lane_off + row * 4, int(cut), kAuxDev);
                        lw[c] = __builtin_amdgcn_raw_buffer_load_b32(prs, lane_off + (16 + row) * 4, int(cut), kAuxDev);
                        p0[c] = __builtin_amdgcn_raw_buffer_load_b128(prs, lane_off + (32 + row * H + ch * 8) * 4, int(cut), kAuxDev);
                        p1[c] = __builtin_amdgcn_raw_buffer_load_b128(prs, lane_off + (32 + row * H + ch * 8) * 4 + 16, int(cut), kAuxDev);
                    }
                    float mnew = mg;
#pragma unroll
                    for (int c = 0; c < CH; ++c)
                        if (s0 + c < S) mnew = fmaxf(mnew, __uint_as_float(mw[c]));
                    const float resc = __builtin_amdgcn_exp2f(mg - mnew);
                    lg *= resc;
#pragma unroll
                    for (int q = 0; q < 8; ++q) v8[q] *= resc;
#pragma unroll
                    for (int c = 0; c < CH; ++c) {
                        const float f = s0 + c < S ? __builtin_amdgcn_exp2f(__uint_as_float(mw[c]) - mnew) : 0.f;
                        lg += f * __uint_as_float(lw[c]);
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            v8[q] += f * __uint_as_float(p0[c][q]);
                            v8[4 + q] += f * __uint_as_float(p1[c][q]);
                        }
                    }
                    mg = mnew;
                }
                if (item) inv_l = 1.0f / lg;
                if (tsp && tid == 0) tsp[31] = wall_clock64();
                if (tid == 0)
                    __hip_atomic_store(&acount[kvh * row_tiles + rt], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (finish && item && rr < R) {
#pragma unroll
            for (int q = 0; q < 8; ++q) v8[q] *= inv_l;
            const int m = rr / G, gl = rr % G;
            const int k0 = (kvh * G + gl) * H + ch * 8;
            st_dev_frag8(attfrag_l, frag_index(k0, m, rp), v8);
        }
}

// Page buffers per wavefront (K and V fragments of one page and head each): as many as the
// register file allows next to the query and output tiles.
template <int H>
struct AttnBufs {
    static constexpr int N = H == 128 ? 2 : 4;  // 64 registers of the consumer's 256
    bf16x8 k[N][H / 32];
    short4v v[N][H / 16];
};

// Before the barrier: issue the loads of the first task's first pages where those hold old
// context only (they do not depend on this layer's QKV phase).  loaded[i] tells the phase.
template <int H>
__device__ __forceinline__ void attn_preload(const MegaArgs& a, int layer, int wave, int lane, int wg, AttnBufs<H>& bf,
                                             const int (&pid)[8], bool (&loaded)[8]) {
    constexpr int NBUF = AttnBufs<H>::N;
#pragma unroll
    for (int i = 0; i < NBUF; ++i) loaded[i] = false;
    if (wg >= a.Hkv * a.row_tiles * a.a_splits) return;
    const AttnTask t = attn_task(a, wg);
    const __bf16* kpool = a.kpool + size_t(layer) * a.pool_layer_elems;
    const __bf16* vpool = a.vpool + size_t(layer) * a.pool_layer_elems;
#pragma unroll
    for (int i = 0; i < NBUF; ++i) {
        const int pg = t.pg0 + wave + i * kMegaWaves;
        loaded[i] = pg < t.pg1 && (pg + 1) * 16 <= a.old_end;
        if (loaded[i]) attn_load_page<H>(a, kpool, vpool, t.kvh, pid[i], lane, bf.k[i], bf.v[i]);
    }
}

// The page ids of a workgroup's first attention task are the same in every layer (one block
// table for all layers): fetched once at kernel start, so that no page load ever waits for an id
// queued behind a phase's stores.
template <int H>
__device__ __forceinline__ void attn_page_ids(const MegaArgs& a, int wave, int wg, int (&pid)[8]) {
    constexpr int NBUF = AttnBufs<H>::N;
#pragma unroll
    for (int i = 0; i < 8; ++i) pid[i] = 0;
    if (wg >= a.Hkv * a.row_tiles * a.a_splits) return;
    const AttnTask t = attn_task(a, wg);
#pragma unroll
    for (int i = 0; i < NBUF; ++i) {
        const int pg = t.pg0 + wave + i * kMegaWaves;
        if (pg < t.pg1) pid[i] = __builtin_amdgcn_readfirstlane(a.block_table[pg]);
    }
}

template <int H, bool TREE>
__device__ __forceinline__ void attn_phase(const MegaArgs& a, int layer, MegaSmem& sm, int wave, int lane, int wg,
                                           AttnBufs<H>& bf, const int (&pid0)[8], bool (&loaded)[8], uint32_t& cgen) {
    constexpr int ST = H / 32, HT = H / 16, PART = 16 * (H + 2), NBUF = AttnBufs<H>::N;
    const int tid = threadIdx.x;
    const int R = a.G * a.r;
    const int col = lane & 15, kq = lane >> 4;
    const __bf16* kpool = a.kpool + size_t(layer) * a.pool_layer_elems;
    const __bf16* vpool = a.vpool + size_t(layer) * a.pool_layer_elems;
    const int n_tasks = a.Hkv * a.row_tiles * a.a_splits;
    for (int task = wg; task < n_tasks; task += a.nwg) {
        const AttnTask t = attn_task(a, task);
        const int kvh = t.kvh, rt = t.rt;
        const int rho = rt * 16 + col;
        const bool row_ok = rho < R;
        const int mrow = row_ok ? rho / a.G : -1;
        const int limit = a.slot0 + mrow;  // chain: last visible slot of this lane's row
        // tree rows: the lane's mask row (rows beyond R read row 0 and are dropped by mrow < 0)
        const uint32_t* mrow_mask = TREE ? a.tmask + size_t(mrow < 0 ? 0 : mrow) * a.tmask_words : nullptr;
        int pg = t.pg0 + wave;
        {
            int pid[NBUF];
            bool need[NBUF];
#pragma unroll
            for (int i = 0; i < NBUF; ++i) {
                const int pgi = pg + i * kMegaWaves;
                need[i] = pgi < t.pg1 && !(task == wg && loaded[i]);
                pid[i] = task == wg ? pid0[i] : (need[i] ? a.block_table[pgi] : 0);
            }
#pragma unroll
            for (int i = 0; i < NBUF; ++i)
                if (need[i]) attn_load_page<H>(a, kpool, vpool, kvh, pid[i], lane, bf.k[i], bf.v[i]);
        }
        bf16x8 qh[ST], ql[ST];
        {
            const bf16x8* qp = reinterpret_cast<const bf16x8*>(
                a.qfrag + size_t(layer) * a.qfrag_stride + ((size_t(kvh) * (a.G * kMaxR) + (row_ok ? rho : 0)) * (H >> 3)) * 16);
#pragma unroll
            for (int st = 0; st < ST; ++st) {
                qh[st] = qp[(st * 4 + kq) * 2];
                ql[st] = qp[(st * 4 + kq) * 2 + 1];
            }
        }
        floatx4 o[HT];
#pragma unroll
        for (int i = 0; i < HT; ++i) o[i] = floatx4{0.f, 0.f, 0.f, 0.f};
        float mx = -1e30f, sum = 0.f;

        // Two pages per round: one max / sum reduction across the lane groups and one rescale of
        // the output tile serve 32 keys.  Scores are in log2 units (the query carries log2(e)/sqrt(h)).
        // `scores_done` runs once the K operands have been consumed: the refill of those registers
        // starts there, a softmax and an output update ahead of the refill of V
        auto use_two = [&](int pga, const bf16x8 (&ka)[ST], const short4v (&va)[HT], int pgb, const bf16x8 (&kb)[ST],
                           const short4v (&vb)[HT], auto&& scores_done) {
            floatx4 sa = floatx4{0.f, 0.f, 0.f, 0.f}, sb = floatx4{0.f, 0.f, 0.f, 0.f};
            // Tree rows (draft side: a node sees the context, its ancestors and itself, never its
            // peers): the 16 visibility bits of each page come from the row's mask word, fetched
            // here and used after the score instructions.  Pages below the mask's base are context.
            uint32_t bits_a = 0xffffu, bits_b = 0xffffu;
            if constexpr (TREE) {
                const int oa = pga * 16 - a.tmask_base, ob = pgb * 16 - a.tmask_base;
                if (oa >= 0) bits_a = (oa >> 5) < a.tmask_words ? (mrow_mask[oa >> 5] >> (oa & 31)) & 0xffffu : 0u;
                if (ob >= 0 && pgb < t.pg1) bits_b = (ob >> 5) < a.tmask_words ? (mrow_mask[ob >> 5] >> (ob & 31)) & 0xffffu : 0u;
            }
#pragma unroll
            for (int st = 0; st < ST; ++st) {
                sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[st], qh[st], sa, 0, 0, 0);
                sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[st], qh[st], sb, 0, 0, 0);
                sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[st], ql[st], sa, 0, 0, 0);
                sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[st], ql[st], sb, 0, 0, 0);
            }
            scores_done();
            float pmax = -1e30f;
            bool oka[4], okb[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if constexpr (TREE) {
                    oka[v] = mrow >= 0 && ((bits_a >> (kq * 4 + v)) & 1u) != 0;
                    okb[v] = mrow >= 0 && pgb < t.pg1 && ((bits_b >> (kq * 4 + v)) & 1u) != 0;
                } else {
                    oka[v] = mrow >= 0 && (pga * 16 + kq * 4 + v) <= limit;
                    okb[v] = mrow >= 0 && pgb < t.pg1 && (pgb * 16 + kq * 4 + v) <= limit;
                }
                if (oka[v]) pmax = fmaxf(pmax, sa[v]);
                if (okb[v]) pmax = fmaxf(pmax, sb[v]);
            }
            pmax = fmaxf(pmax, __shfl_xor(pmax, 16));
            pmax = fmaxf(pmax, __shfl_xor(pmax, 32));
            const float mnew = fmaxf(mx, pmax);
            const float alpha = __builtin_amdgcn_exp2f(mx - mnew);
            float pa[4], pb[4], psum = 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                pa[v] = oka[v] ? __builtin_amdgcn_exp2f(sa[v] - mnew) : 0.f;
                pb[v] = okb[v] ? __builtin_amdgcn_exp2f(sb[v] - mnew) : 0.f;
                psum += pa[v] + pb[v];
            }
            psum += __shfl_xor(psum, 16);
            psum += __shfl_xor(psum, 32);
            sum = sum * alpha + psum;
            mx = mnew;
            short4v pah, pal, pbh, pbl;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                __bf16 hi, lo;
                split_bf16(pa[v], hi, lo);
                pah[v] = __builtin_bit_cast(short, hi);
                pal[v] = __builtin_bit_cast(short, lo);
                split_bf16(pb[v], hi, lo);
                pbh[v] = __builtin_bit_cast(short, hi);
                pbl[v] = __builtin_bit_cast(short, lo);
            }
#pragma unroll
            for (int i = 0; i < HT; ++i) {
                floatx4 acc = o[i];
                acc[0] *= alpha; acc[1] *= alpha; acc[2] *= alpha; acc[3] *= alpha;
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va[i], pah, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vb[i], pbh, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va[i], pal, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vb[i], pbl, acc, 0, 0, 0);
                o[i] = acc;
            }
        };
        if (a.ts && layer == a.ts_layer && tid == 0) a.ts[size_t(wg) * 32 + 13] = wall_clock64();
        // buffers in rotation, two at a time: the others stay in flight behind the pair in use
        static_assert(NBUF % 2 == 0, "pairs");
        int pid_nx[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int nx = pg + (NBUF + q) * kMegaWaves;
            pid_nx[q] = nx < t.pg1 ? a.block_table[nx] : 0;
        }
        while (pg < t.pg1) {
#pragma unroll
            for (int i = 0; i < NBUF; i += 2) {
                if (pg < t.pg1) {
                    use_two(pg, bf.k[i], bf.v[i], pg + kMegaWaves, bf.k[i + 1], bf.v[i + 1], [&]() {
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const int nx = pg + (NBUF + q) * kMegaWaves;
                            if (nx < t.pg1) attn_load_k<H>(a, kpool, kvh, pid_nx[q], lane, bf.k[i + q]);
                        }
                    });
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const int nx = pg + (NBUF + q) * kMegaWaves;
                        if (nx < t.pg1) attn_load_v<H>(a, vpool, kvh, pid_nx[q], lane, bf.v[i + q]);
                    }
                    // ids for the refills after these: behind the page loads in the queue, they will
                    // have arrived a round later
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const int nx2 = pg + (NBUF + 2 + q) * kMegaWaves;
                        pid_nx[q] = nx2 < t.pg1 ? a.block_table[nx2] : 0;
                    }
                }
                pg += 2 * kMegaWaves;
            }
        }

        if (a.ts && layer == a.ts_layer && tid == 0) a.ts[size_t(wg) * 32 + 14] = wall_clock64();
        // wavefront partials -> LDS: M[16], L[16], O[16][H]
        float* mine = sm.attn + wave * PART;
        if (kq == 0) {
            mine[col] = mx;
            mine[16 + col] = sum;
        }
#pragma unroll
        for (int i = 0; i < HT; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) mine[32 + col * H + i * 16 + kq * 4 + v] = o[i][v];
        cbar(sm, cgen);
        if (a.ts && layer == a.ts_layer && tid == 0) a.ts[size_t(wg) * 32 + 15] = wall_clock64();
        attn_finish<H>(sm, a.apart, a.acount, a.attfrag + size_t(layer) * a.attfrag_stride, a.G, a.rp, R, a.a_splits,
                       a.row_tiles, task, t.split, kvh, rt, cgen,
                       (a.ts && layer == a.ts_layer) ? a.ts + size_t(wg) * 32 : nullptr);
        cbar(sm, cgen);
    }
}
// ---- the kernel ----------------------------------------------------------------------------------
// DR: draft-side call (tree rows with a visibility mask, per-row top-k in the vocabulary phase)
template <int MT, int H, bool PK, bool DR>
__global__ __launch_bounds__(kBlockThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_verify(MegaArgs a) {
    __shared__ MegaSmem sm;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wg = blockIdx.x, nwg = a.nwg;
    if (tid == 0) {
        sm.failed = 0;
        sm.cbar = 0;
        sm.epoch = __hip_atomic_load(&a.bar[kBarEpoch], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sm.ws_ok = __hip_atomic_load(&a.bar[kBarMagic], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == kWsMagic;
    }
    if (tid < kMegaWaves) sm.tail[tid] = sm.head[tid] = 0;
    if (tid < kMaxR) sm.wg_best[tid] = 0ull;
    __syncthreads();  // the only hardware barrier: producers and consumers part ways here
    // A workspace whose control words were never prepared could hold flags that let barriers fall
    // through: every workgroup reads the same word, so all of them leave, and the step fails.
    if (!sm.ws_ok) {
        if (wg == 0 && tid == 0) {
            a.out->accepted_len = -1;
            a.out->correction_token = -1;
            a.out->kv_first_slot = a.ctx_len;
            a.out->kv_count = 0;
        }
        return;
    }

    if (wave >= kMegaWaves) {
        producer<!PK>(a, sm, wave - kMegaWaves, lane, wg);
        return;
    }

    uint32_t gen = 0, cgen = 0;
    FifoC fc = {0u, 0u, 0u, false, 0u};
    const int n_dt = a.d >> 4;  // 16-column tiles of the residual stream
    auto layer_base = [&](int l) { return a.wbase + a.layer0_off + size_t(l) * a.layer_stride; };

    // ---- embed: x0 = E[token], its gained high/low fragments, per-tile sums of squares ----
    {
        const __bf16* E = reinterpret_cast<const __bf16*>(a.wbase + a.embed_off);
        const float* g0 = reinterpret_cast<const float*>(layer_base(0) + a.g_attn_off);
        constexpr int TP = kMegaThreads / (2 * kMaxR);  // tiles per pass
        const int c = tid & 1, m = (tid >> 1) % kMaxR, i = tid / (2 * kMaxR);
        for (int t = wg * TP + i; t < n_dt; t += nwg * TP) {
            float ssum = 0.f;
            const bool on = m < a.r;
            if (on) {
                int tok = a.cand[m];
                tok = tok < 0 ? 0 : (tok >= a.V ? a.V - 1 : tok);
                const int n0 = t * 16 + c * 8;
                const bf16x8 ev = *reinterpret_cast<const bf16x8*>(E + size_t(tok) * a.d + n0);
                float nv[8], gv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    nv[e] = static_cast<float>(ev[e]);
                    ssum += nv[e] * nv[e];
                    gv[e] = nv[e] * g0[n0 + e];
                }
                st_dev_f32x8(a.xres, uint32_t(m) * a.d + n0, nv);
                st_dev_frag8(a.xfrag, frag_index(n0, m, a.rp), gv);
            }
            ssum += __shfl_xor(ssum, 1);
            if (on && c == 0) st_agent(a.ss + size_t(m) * n_dt + t, ssum);
        }
        // rotation table in fp64 (long contexts stay exact), spread over the grid
        const int half = a.h >> 1;
        for (int e = wg * kMegaThreads + tid; e < a.r * half; e += nwg * kMegaThreads) {
            const int m2 = e / half, j = e % half;
            const double ang = double(a.row_pos ? a.row_pos[m2] : a.ctx_len + m2) * pow(double(a.theta), -2.0 * j / a.h);
            st_agent(a.rope + m2 * half + j, float(cos(ang)));
            st_agent(a.rope + kMaxR * half + m2 * half + j, float(sin(ang)));
        }
        if (wg == 0 && tid < kMaxR)
            __hip_atomic_store(&a.best[tid], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    store_wait();
    grid_wait(a, gen, sm, cgen);

    int pid0[8];
    attn_page_ids<H>(a, wave, wg, pid0);
    const size_t xres_stride = size_t(kMaxR) * a.d, ss_stride = size_t(n_dt) * kMaxR;
#define CARD_TS(i)                                                                  \
    if (a.ts && l == a.ts_layer && tid == 0) a.ts[size_t(wg) * 32 + (i)] = wall_clock64();
    for (int l = 0; l < a.L; ++l) {
        const char* lb = layer_base(l);
        const int v0 = 2 * l, v1 = 2 * l + 1, v2 = 2 * l + 2;
        const bool last = l + 1 == a.L;
        EpiArgs ea = {};
        ea.layer = l;
        
        // QKV (+norm scale, rotation, KV write).  Pages that hold only old context do not depend
        // on this phase: their loads are issued as soon as the k-loop is over, ahead of the
        // epilogue's stores, and land while the barrier in front of attention is crossed.
        const PhasePlan p_qkv = stream_phase<!PK>(a, 4 * l + SP_QKV, wg, wave);
        ea.ss_in = a.ss + v0 * ss_stride;
        ea.qfrag = a.qfrag + size_t(l) * a.qfrag_stride;
        ea.kpool = a.kpool + size_t(l) * a.pool_layer_elems;
        ea.vpool = a.vpool + size_t(l) * a.pool_layer_elems;
        AttnBufs<H> bf;
        bool loaded[8];
        auto preload = [&]() {
            CARD_TS(11)
            // a pair's second page may not exist: its probabilities are zero, its buffer must be finite
#pragma unroll
            for (int i = 0; i < AttnBufs<H>::N; ++i) {
#pragma unroll
                for (int q = 0; q < H / 32; ++q) bf.k[i][q] = __builtin_bit_cast(bf16x8, uint4v{0u, 0u, 0u, 0u});
#pragma unroll
                for (int q = 0; q < H / 16; ++q) bf.v[i][q] = short4v{0, 0, 0, 0};
            }
            attn_preload<H>(a, l, wave, lane, wg, bf, pid0, loaded);
            CARD_TS(16)
        };
        CARD_TS(0)
        ea.ts0 = 21;
        gemm_phase<kNbQkv, MT, ME_QKV, PK>(a, p_qkv, a.xfrag + v0 * a.xfrag_stride, uint32_t(a.xfrag_stride * 2), ea, fc,
                                          sm, wave, lane, cgen, preload);
        CARD_TS(1)
        store_wait();
        CARD_TS(12)
        grid_wait(a, gen, sm, cgen);
        CARD_TS(2)
        attn_phase<H, DR>(a, l, sm, wave, lane, wg, bf, pid0, loaded, cgen);
        CARD_TS(3)
        store_wait();
        grid_wait(a, gen, sm, cgen);
        CARD_TS(4)

        // O-projection + residual -> version v1, gained with the FFN norm's gain
        const PhasePlan p_wo = stream_phase<!PK>(a, 4 * l + SP_WO, wg, wave);
        ea.xres_old = a.xres + v0 * xres_stride;
        ea.xres_new = a.xres + v1 * xres_stride;
        ea.xfrag_new = a.xfrag + v1 * a.xfrag_stride;
        ea.ss_new = a.ss + v1 * ss_stride;
        ea.gain_next = reinterpret_cast<const float*>(lb + a.g_ffn_off);
        ea.ts0 = 24;
        gemm_phase<kNbOne, MT, ME_RESID, PK>(a, p_wo, a.attfrag + size_t(l) * a.attfrag_stride,
                                            uint32_t(a.attfrag_stride * 2), ea, fc, sm, wave, lane, cgen);
        CARD_TS(5)
        store_wait();
        grid_wait(a, gen, sm, cgen);
        CARD_TS(6)

        // gate/up + SwiGLU
        const PhasePlan p_gu = stream_phase<!PK>(a, 4 * l + SP_GU, wg, wave);
        ea.ss_in = a.ss + v1 * ss_stride;
        ea.actfrag = a.actfrag + size_t(l) * a.actfrag_stride;
        ea.ts0 = 0;
        gemm_phase<kNbWide, MT, ME_SWIGLU, PK>(a, p_gu, a.xfrag + v1 * a.xfrag_stride, uint32_t(a.xfrag_stride * 2), ea,
                                              fc, sm, wave, lane, cgen);
        CARD_TS(7)
        store_wait();
        grid_wait(a, gen, sm, cgen);
        CARD_TS(8)

        // down + residual -> version v2, gained with the next norm's gain
        const PhasePlan p_wd = stream_phase<!PK>(a, 4 * l + SP_WD, wg, wave);
        ea.xres_old = a.xres + v1 * xres_stride;
        ea.xres_new = a.xres + v2 * xres_stride;
        ea.xfrag_new = a.xfrag + v2 * a.xfrag_stride;
        ea.ss_new = a.ss + v2 * ss_stride;
        ea.gain_next = last ? reinterpret_cast<const float*>(a.wbase + a.g_final_off)
                            : reinterpret_cast<const float*>(layer_base(l + 1) + a.g_attn_off);
        ea.ts0 = 27;
        if constexpr (!PK) {
            if (down_grouped(a))
                gemm_phase<4, MT, ME_RESID, false, NoHook, true>(a, p_wd, a.actfrag + size_t(l) * a.actfrag_stride,
                                                                 uint32_t(a.actfrag_stride * 2), ea, fc, sm, wave, lane, cgen);
            else
                gemm_phase<kNbOne, MT, ME_RESID, false>(a, p_wd, a.actfrag + size_t(l) * a.actfrag_stride,
                                                        uint32_t(a.actfrag_stride * 2), ea, fc, sm, wave, lane, cgen);
        } else {
            gemm_phase<kNbOne, MT, ME_RESID, PK>(a, p_wd, a.actfrag + size_t(l) * a.actfrag_stride,
                                                uint32_t(a.actfrag_stride * 2), ea, fc, sm, wave, lane, cgen);
        }
        CARD_TS(9)
        store_wait();
        grid_wait(a, gen, sm, cgen);
        CARD_TS(10)
    }

    // vocabulary head + arg-max
    {
                const PhasePlan p_lm = stream_phase<!PK>(a, 4 * a.L, wg, wave);
        EpiArgs ea = {};
        ea.ss_in = a.ss + size_t(2 * a.L) * ss_stride;
        LmState lm = {{0ull, 0ull}, -1e30f, 0.f};
        ea.lm = &lm;
        gemm_phase<kNbWide, MT, DR ? ME_LM_TOPK : ME_LM, PK>(a, p_lm, a.xfrag + size_t(2 * a.L) * a.xfrag_stride,
                                          uint32_t(a.xfrag_stride * 2), ea, fc, sm, wave, lane, cgen);
        if (tid < a.r && sm.wg_best[tid] != 0ull)
            __hip_atomic_fetch_max(&a.best[tid], sm.wg_best[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if constexpr (DR) {
            // this workgroup's share of every row: its sixteen best keys and its (max, sum of exp)
            constexpr int LPR = kMegaThreads / (16 * MT), RUN = 16 / LPR;
            const int m = tid / LPR, p = tid % LPR;
            float mx = lm.m;
#pragma unroll
            for (int o = 1; o < LPR; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
            float sx = lm.s * __expf(lm.m - mx);
#pragma unroll
            for (int o = 1; o < LPR; o <<= 1) sx += __shfl_xor(sx, o);
            if (m < a.r) {
                unsigned long long* dst = a.topk_part + (size_t(wg) * kMaxR + m) * 16;
#pragma unroll
                for (int u = 0; u < RUN; ++u)
                    __hip_atomic_store(dst + u * LPR + p, lm.run[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (p == 0) {
                    st_agent(a.lse_part + (size_t(wg) * kMaxR + m) * 2, mx);
                    st_agent(a.lse_part + (size_t(wg) * kMaxR + m) * 2 + 1, sx);
                }
            }
        }
    }
    store_wait();
    grid_wait(a, gen, sm, cgen);

    if constexpr (DR) {
        // Rows are merged by one workgroup each: thread t holds workgroup t's sorted list of sixteen
        // keys for the row and its (max, sum) pair; the log-sum-exp folds the pairs, then k rounds of
        // "largest list head in the workgroup" emit the row's k best tokens with their probabilities.
        for (int m = wg; m < a.r; m += nwg) {
            unsigned long long mine[16];
            float pm = -1e30f, ps = 0.f;
            if (tid < nwg) {
                const unsigned long long* src = a.topk_part + (size_t(tid) * kMaxR + m) * 16;
#pragma unroll
                for (int j = 0; j < 16; ++j) mine[j] = __hip_atomic_load(src + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                pm = ld_agent(a.lse_part + (size_t(tid) * kMaxR + m) * 2);
                ps = ld_agent(a.lse_part + (size_t(tid) * kMaxR + m) * 2 + 1);
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j) mine[j] = 0ull;
            }
            float* red = sm.wgt;  // [0..3] maxima, [4..7] sums of the four consumer wavefronts
            float mx = pm;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
            if (lane == 0) red[wave] = mx;
            cbar(sm, cgen);
            mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
            float sx = ps * __expf(pm - mx);
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) sx += __shfl_xor(sx, o);
            if (lane == 0) red[4 + wave] = sx;
            cbar(sm, cgen);
            const float lse = mx + __logf((red[4] + red[5]) + (red[6] + red[7]));
            for (int j = 0; j < a.topk; ++j) {
                unsigned long long best = mine[0];
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const unsigned long long other = __shfl_xor(best, o);
                    best = other > best ? other : best;
                }
                unsigned long long* slot = sm.part_best + (j & 1) * kMegaWaves;
                if (lane == 0) slot[wave] = best;
                cbar(sm, cgen);
                best = slot[0];
#pragma unroll
                for (int w2 = 1; w2 < kMegaWaves; ++w2) best = slot[w2] > best ? slot[w2] : best;
                if (best != 0ull && mine[0] == best) {
#pragma unroll
                    for (int i = 0; i < 15; ++i) mine[i] = mine[i + 1];
                    mine[15] = 0ull;
                }
                if (tid == 0) {
                    const uint32_t kb = uint32_t(best >> 32);
                    const float logit = __uint_as_float((kb & 0x80000000u) ? (kb & 0x7fffffffu) : ~kb);
                    a.topk_tok[m * a.topk + j] = best != 0ull ? int(0xffffffffu - uint32_t(best & 0xffffffffull)) : -1;
                    a.topk_prob[m * a.topk + j] = best != 0ull ? __expf(logit - lse) : 0.f;
                }
            }
            cbar(sm, cgen);
        }
    }
    if (wg == 0) {
        if (tid < a.r) {
            const unsigned long long k = __hip_atomic_load(&a.best[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sm.pred[tid + 1] = int(0xffffffffu - uint32_t(k & 0xffffffffull));
        }
        cbar(sm, cgen);
        if (tid == 0) {
            sm.pred[0] = a.pending < 0 ? a.cand[0] : a.pending;
            int j = 0;
            while (j < a.r && a.cand[j] == sm.pred[j]) ++j;
            // weights laid out for another grid size would stream in the wrong order
            const bool bad_layout = a.stamp[0] != kStampMagic || a.stamp[1] != uint32_t(nwg);
            // a token id outside the vocabulary was clamped by the embedding gather: the step is void
            bool bad_token = false;
            for (int i = 0; i < a.r; ++i) bad_token = bad_token || a.cand[i] < 0 || a.cand[i] >= a.V;
            const bool failed = bad_layout || bad_token || sm.failed ||
                                __hip_atomic_load(&a.bar[kBarError], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
            a.out->accepted_len = failed ? -1 : j;
            a.out->correction_token = failed ? -1 : sm.pred[j];
            a.out->kv_first_slot = a.ctx_len;
            a.out->kv_count = failed ? 0 : j;
        }
        if (a.row_argmax && tid < a.r) a.row_argmax[tid] = sm.pred[tid + 1];
    }
    // the last workgroup to leave re-arms the counters for the next call
    if (tid == 0) {
        const uint32_t prev = __hip_atomic_fetch_add(&a.bar[kBarExit], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (prev == uint32_t(nwg) - 1) {
            // barrier sequence numbers of the next call start above anything this call used
            __hip_atomic_store(&a.bar[kBarEpoch], sm.epoch + 8192u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&a.bar[kBarExit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&a.bar[kBarError], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}


}  // namespace card
