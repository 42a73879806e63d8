// C ABI of libllsa: host-side plan (validation, level table, buffer layout) and the launch sequences of
// the forward and backward passes.  No device memory is allocated here and the host never waits.
#include <math.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "llsa_internal.h"

namespace llsa {

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

LevelTable make_level_table(const Plan &p, const void *K0, const void *V0, const int32_t *indices,
                            const void *workspace) {
    LevelTable t;
    memset(&t, 0, sizeof(t));
    const char *w = static_cast<const char *>(workspace);
    const char *idx = reinterpret_cast<const char *>(indices);
    int64_t bp = 1;
    int pos = 0, bpos = 0;
    for (int l = 0; l <= p.L; ++l) {
        t.K[l] = (l == 0) ? K0 : (const void *)(w + p.pyr_off[1][l]);
        t.V[l] = (l == 0) ? V0 : (const void *)(w + p.pyr_off[2][l]);
        t.I[l] = (l < p.L) ? reinterpret_cast<const int32_t *>(idx + p.idx_off[l]) : nullptr;
        t.n[l] = p.n[l];
        t.rows[l] = (l < p.L) ? p.n[l + 1] : 0;
        t.Kl[l] = (l < p.L) ? p.Kl[l] : 0;
        t.Bpow[l] = bp;
        t.bias[l] = p.desc.reweight ? (float)(l * log((double)p.B)) : 0.f;
        if (l <= p.Le) {
            t.seg[l] = pos;
            pos += (l < p.L) ? p.Kl[l] * p.B : (int)p.n[l];
            t.bseg[l] = bpos;
            bpos += (l < p.L) ? p.Kl[l] * ((p.B + 15) / 16) : (int)((p.n[l] + 15) / 16);
        }
        bp *= p.B;
    }
    t.Bpow[p.L + 1] = bp;
    t.nlev = p.Le + 1;
    t.seg[t.nlev] = pos;
    t.bseg[t.nlev] = bpos;
    t.L = p.L;
    t.B = p.B;
    t.lb = p.lb;
    t.ls = p.lb >= 4 ? p.lb - 4 : 0;
    t.d = p.d;
    t.scale = p.scale;
    return t;
}

static llsa_status build_plan(const llsa_desc &d, Plan &p) {
    memset(&p, 0, sizeof(p));
    p.desc = d;
    if (d.batch < 1 || d.heads < 1 || d.N < 1 || d.K < 1 || d.L < 1 || d.B < 2) return LLSA_ERR_BAD_SHAPE;
    if (d.Le < 0 || d.Le > d.L) return LLSA_ERR_BAD_SHAPE;
    if (d.dtype != LLSA_F32 && d.dtype != LLSA_BF16) return LLSA_ERR_UNSUPPORTED;
    if (d.d != 16 && d.d != 32 && d.d != 64 && d.d != 128) return LLSA_ERR_UNSUPPORTED;
    if (d.B > 64 || d.K > 64 || d.L > kMaxL) return LLSA_ERR_UNSUPPORTED;
    if (d.N > ((int64_t)1 << 30) || (int64_t)d.batch * d.heads > (1 << 20)) return LLSA_ERR_UNSUPPORTED;
    // launch grids are 32-bit counts of workgroups (at least 16 tokens each) and the key-major lists use 32-bit offsets
    if ((int64_t)d.batch * d.heads * ((d.N + 15) / 16) >= ((int64_t)1 << 31)) return LLSA_ERR_UNSUPPORTED;
    if ((d.N / d.B) * (int64_t)(d.K < d.N / d.B ? d.K : d.N / d.B) >= ((int64_t)1 << 31)) return LLSA_ERR_UNSUPPORTED;
    int64_t bl = 1;
    for (int l = 0; l < d.L; ++l) {
        bl *= d.B;
        if (bl > d.N) return LLSA_ERR_BAD_SHAPE;
    }
    if (d.N % bl != 0) return LLSA_ERR_BAD_SHAPE;
    p.L = d.L; p.Le = d.Le; p.B = d.B; p.K = d.K; p.d = d.d; p.N = d.N;
    p.bh = d.batch * d.heads;
    p.elt = d.dtype == LLSA_F32 ? 4 : 2;
    p.scale = d.sm_scale > 0.f ? d.sm_scale : (float)(1.0 / sqrt((double)d.d));
    int64_t nl = d.N;
    for (int l = 0; l <= p.L; ++l) { p.n[l] = nl; nl /= d.B; }
    size_t off = 0;
    for (int l = 0; l < p.L; ++l) {
        p.Kl[l] = (int)(p.n[l + 1] < d.K ? p.n[l + 1] : d.K);
        p.idx_off[l] = off;
        off += (size_t)p.bh * p.n[l + 1] * p.Kl[l] * sizeof(int32_t);
    }
    p.idx_bytes = off;
    // MFMA kernels: bf16, blocks of 1, 2 or 4 16-token tiles, d = 64 / 128, and whole workgroups of 4 query tiles per head
    p.fast = d.kernel_path == 0 && d.dtype == LLSA_BF16 && (d.B == 16 || d.B == 32 || d.B == 64) &&
             (d.d == 64 || d.d == 128) && d.N % 64 == 0;
    p.lb = !p.fast ? 0 : d.B == 16 ? 4 : d.B == 32 ? 5 : 6;
    // the portable selection holds one row of candidate scores per wave in LDS (the fast one takes any number)
    for (int l = 1; l <= p.L; ++l) {
        const int64_t cand = (l == p.L) ? p.n[l] : (int64_t)p.Kl[l] * p.B;
        if (cand > kMaxCand && !select_fast_ok(p, l)) return LLSA_ERR_UNSUPPORTED;
    }
    int64_t m = 0;
    for (int l = 0; l <= p.Le; ++l) m += (l < p.L) ? (int64_t)p.Kl[l] * p.B : p.n[l];
    p.list_len = (int)m;

    // ---- workspace: pooled levels first (shared by forward and backward) ----
    size_t ws = 0;
    for (int x = 0; x < 3; ++x)
        for (int l = 1; l <= p.L; ++l) {
            p.pyr_off[x][l] = ws;
            ws = align_up(ws + (size_t)p.bh * p.n[l] * p.d * p.elt);
        }
    p.ws_fwd = ws;
    p.D_off = ws;
    ws = align_up(ws + (size_t)p.bh * p.N * sizeof(float));
    for (int l = 0; l < p.L; ++l) {
        const size_t keys = (size_t)p.bh * p.n[l + 1], ent = keys * p.Kl[l];
        p.C_off[l] = ws;     ws = align_up(ws + ((size_t)p.bh * (p.n[l + 1] + 1)) * sizeof(int32_t));
        p.cnt_off[l] = ws;   ws = align_up(ws + keys * sizeof(int32_t));
        p.Iq_off[l] = ws;    ws = align_up(ws + ent * sizeof(int32_t));
        p.Iqtmp_off[l] = ws; ws = align_up(ws + ent * sizeof(int32_t));
    }
    for (int l = 1; l <= p.L; ++l) {
        const size_t bytes = (size_t)p.bh * p.n[l] * p.d * sizeof(float);
        p.dKacc_off[l] = ws; ws = align_up(ws + bytes);
        p.dVacc_off[l] = ws; ws = align_up(ws + bytes);
    }
    // coarse-level dK/dV grouped by level-1 query block: d = 64, whole groups of 256 queries, short lists
    int coarse_blocks = 0;
    for (int l = 1; l <= dkv_group_top(p); ++l) coarse_blocks += (l < p.L) ? p.Kl[l] : (int)((p.n[l] + 15) / 16);
    p.group = p.fast && d.B == 16 && d.N % 256 == 0 && p.Le >= 1 && coarse_blocks <= 512 && dkv_group_top(p) >= 1;
    p.grp_slab_off = p.grp_red_off[0] = p.grp_red_off[1] = ws;
    if (p.group) {
        size_t slab = 0, red = 0;
        dkv_group_sizes(p, &slab, &red);
        p.grp_slab_off = ws;   ws = align_up(ws + slab);
        p.grp_red_off[0] = ws; ws = align_up(ws + red);
        p.grp_red_off[1] = ws; ws = align_up(ws + red);
    }
    p.part_off = ws;
    p.part_bytes = 0;
    if (p.fast)
        for (int l = p.group ? dkv_group_top(p) + 1 : 1; l <= p.Le; ++l) {   // split slabs of the key-major kernels
            const size_t slab = (size_t)p.bh * ((p.n[l] + 15) / 16) * 16 * p.d * sizeof(float);
            const size_t need = 2 * slab * dkv_splits(p, l);
            if (need > p.part_bytes) p.part_bytes = need;
        }
    ws = align_up(ws + p.part_bytes);
    p.ws_bwd = ws;
    return LLSA_OK;
}

// ---- optional stage timing (benchmark aid) ----
enum Stage { kPool = 0, kSelect, kAttnFwd, kBwdPre, kTranspose, kDq, kDkvCoarse, kUnpool, kDkvFine, kStages };
static const char *const kStageNames[kStages] = {"pool", "select", "attn_fwd", "bwd_pre", "index_transpose",
                                                 "dq", "dkv_coarse", "unpool", "dkv_fine"};
struct StageTimer {
    bool on = false;
    int filter = -1, max_calls = 0, fwd_calls = 0, bwd_calls = 0;
    std::vector<hipEvent_t> ev;          // [max_calls][kStages][2]
    std::vector<unsigned char> rec;      // [max_calls][kStages]: 1 = begin recorded, 2 = both
};
static StageTimer g_timer;

// Brackets one stage of one call; does nothing unless timing is on.
struct StageScope {
    hipEvent_t end = nullptr;
    hipStream_t s;
    unsigned char *flag = nullptr;
    StageScope(int stage, int call, hipStream_t stream) : s(stream) {
        StageTimer &t = g_timer;
        if (!t.on || call >= t.max_calls || (t.filter >= 0 && t.filter != stage)) return;
        const size_t i = (size_t)call * kStages + stage;
        if (hipEventRecord(t.ev[2 * i], s) != hipSuccess) return;
        end = t.ev[2 * i + 1];
        flag = &t.rec[i];
        *flag = 1;
    }
    ~StageScope() {
        if (end && hipEventRecord(end, s) == hipSuccess) *flag = 2;
    }
};

}  // namespace llsa

using namespace llsa;

// The plan's auxiliary stream and the events that fork work onto it and join it back.
struct Aux {
    std::mutex mu;                       // one llsa_backward enqueue sequence per plan at a time
    bool tried = false, ok = false;
    int device = -1;
    hipStream_t side = nullptr;
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};   // fork (the side stream may start), end of the side stream's work (lists ready; join), coarse partials written
};

struct llsa_plan_s {
    Plan p;
    mutable Aux aux;
};

// The auxiliary stream if this call may use it: created at the first call that is not under stream capture
// (nothing may be created while the caller's stream records a graph); later calls reuse it, also under capture.
static Aux *aux_for_call(const llsa_plan_s *plan, hipStream_t s) {
    Aux &a = plan->aux;
    if (plan->p.desc.single_stream || !plan->p.fast) return nullptr;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return nullptr;
    if (!a.tried) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(s, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return nullptr;
        a.tried = true;
        a.device = dev;
        bool ok = hipStreamCreateWithFlags(&a.side, hipStreamNonBlocking) == hipSuccess;
        for (int i = 0; ok && i < 3; ++i) ok = hipEventCreateWithFlags(&a.ev[i], hipEventDisableTiming) == hipSuccess;
        a.ok = ok;
    }
    return (a.ok && a.device == dev) ? &a : nullptr;
}

// ---- forward pass for callers that cannot allocate: the workspace is a static device array ----
// One copy of the array exists on every GPU the library's code object is loaded on, at an address of its own;
// in host code the array's name is only a handle for hipGetSymbolAddress, never a device address.
constexpr size_t kStaticWorkspaceBytes = (size_t)LLSA_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices];     // device address of `scratch` on device i, once looked up there

// Address of the current device's copy of `scratch` (looked up once per device, with that device current).
static llsa_status static_workspace(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return LLSA_ERR_RUNTIME;
    if (dev < 0 || dev >= kMaxDevices) return LLSA_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LLSA_ERR_RUNTIME;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return LLSA_OK;
}

// Every kernel moves 16-byte vectors and the workspace layout assumes a 256-byte aligned base.
static bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
template <class... P> static bool any_misaligned16(P... ptrs) { return (misaligned(ptrs, 16) || ...); }

extern "C" {

llsa_status llsa_plan(const llsa_desc *desc, llsa_plan_t **out) {
    if (!desc || !out) return LLSA_ERR_NULL;
    *out = nullptr;
    Plan p;
    llsa_status st = build_plan(*desc, p);
    if (st != LLSA_OK) return st;
    llsa_plan_s *h = new (std::nothrow) llsa_plan_s;
    if (!h) return LLSA_ERR_RUNTIME;
    h->p = p;
    *out = h;
    return LLSA_OK;
}

void llsa_plan_destroy(llsa_plan_t *plan) {
    if (!plan) return;
    for (hipEvent_t e : plan->aux.ev)
        if (e) (void)hipEventDestroy(e);
    if (plan->aux.side) (void)hipStreamDestroy(plan->aux.side);   // returns at once; pending work still completes
    delete plan;
}

size_t llsa_plan_workspace_bytes(const llsa_plan_t *plan, int for_backward) {
    if (!plan) return 0;
    return for_backward ? plan->p.ws_bwd : plan->p.ws_fwd;
}

size_t llsa_plan_indices_bytes(const llsa_plan_t *plan) { return plan ? plan->p.idx_bytes : 0; }

int32_t llsa_plan_level_info(const llsa_plan_t *plan, int32_t l, int64_t *rows, int32_t *K_l, size_t *byte_offset) {
    if (!plan || l < 0 || l >= plan->p.L) return -1;
    if (rows) *rows = plan->p.n[l + 1];
    if (K_l) *K_l = plan->p.Kl[l];
    if (byte_offset) *byte_offset = plan->p.idx_off[l];
    return plan->p.L;
}

int32_t llsa_plan_pyramid_info(const llsa_plan_t *plan, int32_t tensor, int32_t l, int64_t *tokens,
                               size_t *byte_offset) {
    if (!plan || tensor < 0 || tensor > 2 || l < 1 || l > plan->p.L) return -1;
    if (tokens) *tokens = plan->p.n[l];
    if (byte_offset) *byte_offset = plan->p.pyr_off[tensor][l];
    return 0;
}

int32_t llsa_plan_csc_info(const llsa_plan_t *plan, int32_t l, size_t *C_byte_offset, size_t *Iq_byte_offset) {
    if (!plan || l < 0 || l >= plan->p.L) return -1;
    if (C_byte_offset) *C_byte_offset = plan->p.C_off[l];
    if (Iq_byte_offset) *Iq_byte_offset = plan->p.Iq_off[l];
    return 0;
}

#define LLSA_TRY(expr)                                   \
    do {                                                 \
        if ((expr) != hipSuccess) return LLSA_ERR_RUNTIME; \
    } while (0)
#define LLSA_TRY_ST(expr)                                \
    do {                                                 \
        const llsa_status st_ = (expr);                  \
        if (st_ != LLSA_OK) return st_;                  \
    } while (0)


llsa_status llsa_pool(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, void *workspace,
                      void *hip_stream) {
    if (!plan || !Q || !K || !V || !workspace) return LLSA_ERR_NULL;
    if (any_misaligned16(Q, K, V) || misaligned(workspace, 256)) return LLSA_ERR_BAD_SHAPE;
    LLSA_TRY(launch_pool(plan->p, Q, K, V, workspace, true, (hipStream_t)hip_stream));
    return LLSA_OK;
}

llsa_status llsa_select_level(const llsa_plan_t *plan, int32_t l, const void *workspace, const int32_t *parent,
                              int32_t *out, void *hip_stream) {
    if (!plan || !workspace || !out) return LLSA_ERR_NULL;
    if (l < 1 || l > plan->p.L) return LLSA_ERR_BAD_SHAPE;
    if (l < plan->p.L && !parent) return LLSA_ERR_NULL;
    if (any_misaligned16(parent, out) || misaligned(workspace, 256)) return LLSA_ERR_BAD_SHAPE;
    LLSA_TRY(launch_select(plan->p, l, workspace, parent, out, (hipStream_t)hip_stream));
    return LLSA_OK;
}

llsa_status llsa_attention(const llsa_plan_t *plan, const void *Q, const void *K, const void *V,
                           const int32_t *indices, const void *workspace, void *O, float *LSE, void *hip_stream) {
    if (!plan || !Q || !K || !V || !indices || !workspace || !O || !LSE) return LLSA_ERR_NULL;
    if (any_misaligned16(Q, K, V, O, LSE, indices) || misaligned(workspace, 256)) return LLSA_ERR_BAD_SHAPE;
    const Plan &p = plan->p;
    LevelTable t = make_level_table(p, K, V, indices, workspace);
    if (p.fast) LLSA_TRY(launch_attn_fwd_mfma(p, t, Q, O, LSE, (hipStream_t)hip_stream));
    else LLSA_TRY(launch_attn_fwd_generic(p, t, Q, O, LSE, (hipStream_t)hip_stream));
    return LLSA_OK;
}

static llsa_status forward_impl(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, void *O, float *LSE,
                                int32_t *indices, void *workspace, void *hip_stream, bool pool);

llsa_status llsa_forward(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, void *O, float *LSE,
                         int32_t *indices, void *workspace, void *hip_stream) {
    if (!plan || !Q || !K || !V || !O || !LSE || !indices || !workspace) return LLSA_ERR_NULL;
    if (any_misaligned16(Q, K, V, O, LSE, indices) || misaligned(workspace, 256)) return LLSA_ERR_BAD_SHAPE;
    return forward_impl(plan, Q, K, V, O, LSE, indices, workspace, hip_stream, true);
}

llsa_status llsa_forward_pooled(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, void *O, float *LSE,
                                int32_t *indices, void *workspace, void *hip_stream) {
    if (!plan || !Q || !K || !V || !O || !LSE || !indices || !workspace) return LLSA_ERR_NULL;
    if (any_misaligned16(Q, K, V, O, LSE, indices) || misaligned(workspace, 256)) return LLSA_ERR_BAD_SHAPE;
    return forward_impl(plan, Q, K, V, O, LSE, indices, workspace, hip_stream, false);
}

llsa_status llsa_qknorm_rope_pool(const llsa_plan_t *plan, const void *Qpre, const void *Kpre, const void *V,
                                  const float *gamma_q, const float *gamma_k, const float *cos_table,
                                  const float *sin_table, float eps, void *Qout, void *Kout, void *workspace,
                                  void *hip_stream) {
    if (!plan || !Qpre || !Kpre || !V || !gamma_q || !gamma_k || !cos_table || !sin_table || !Qout || !Kout || !workspace)
        return LLSA_ERR_NULL;
    if (any_misaligned16(Qpre, Kpre, V, Qout, Kout, cos_table, sin_table) || misaligned(workspace, 256))
        return LLSA_ERR_BAD_SHAPE;
    if (!(eps >= 0.f)) return LLSA_ERR_BAD_SHAPE;
    LLSA_TRY(launch_qknorm_rope_pool(plan->p, Qpre, Kpre, V, gamma_q, gamma_k, cos_table, sin_table, eps, Qout, Kout,
                                     workspace, (hipStream_t)hip_stream));
    return LLSA_OK;
}

static llsa_status forward_impl(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, void *O, float *LSE,
                                int32_t *indices, void *workspace, void *hip_stream, bool pool) {
    const Plan &p = plan->p;
    hipStream_t s = (hipStream_t)hip_stream;
    const int call = g_timer.on ? g_timer.fwd_calls++ : 0;
    if (pool) {
        StageScope sc(kPool, call, s);
        LLSA_TRY(launch_pool(p, Q, K, V, workspace, true, s));
    }
    {
        StageScope sc(kSelect, call, s);
        char *idx = reinterpret_cast<char *>(indices);
        int l = p.L;
        if (select_top_fused(p)) {                          // levels L and L-1 in one launch
            LLSA_TRY(launch_select_fast(p, p.L - 1, workspace, nullptr, reinterpret_cast<int32_t *>(idx + p.idx_off[p.L - 2]), s,
                                        reinterpret_cast<int32_t *>(idx + p.idx_off[p.L - 1])));
            l = p.L - 2;
        }
        for (; l >= 1; --l) {
            const int32_t *parent = (l < p.L) ? reinterpret_cast<const int32_t *>(idx + p.idx_off[l]) : nullptr;
            LLSA_TRY(launch_select(p, l, workspace, parent, reinterpret_cast<int32_t *>(idx + p.idx_off[l - 1]), s));
        }
    }
    StageScope sc(kAttnFwd, call, s);
    return llsa_attention(plan, Q, K, V, indices, workspace, O, LSE, hip_stream);
}

// ---- forward pass for callers that cannot allocate (workspace: the static device array above) ----
size_t llsa_static_workspace_bytes(void) { return kStaticWorkspaceBytes; }

llsa_status llsa_forward_static(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, void *O,
                                float *LSE, int32_t *indices, void *hip_stream) {
    if (!plan || !Q || !K || !V || !O || !LSE || !indices) return LLSA_ERR_NULL;
    if (plan->p.ws_fwd > kStaticWorkspaceBytes) return LLSA_ERR_WORKSPACE;     // host-side, before any HIP call
    void *ws = nullptr;
    const llsa_status st = static_workspace(&ws);
    if (st != LLSA_OK) return st;
    return llsa_forward(plan, Q, K, V, O, LSE, indices, ws, hip_stream);
}

llsa_status llsa_index_transpose(const llsa_plan_t *plan, const int32_t *indices, void *workspace, void *hip_stream) {
    if (!plan || !indices || !workspace) return LLSA_ERR_NULL;
    if (any_misaligned16(indices) || misaligned(workspace, 256)) return LLSA_ERR_BAD_SHAPE;
    const Plan &p = plan->p;
    LLSA_TRY(launch_csc(p, p.L - 1, indices, workspace, (hipStream_t)hip_stream));
    return LLSA_OK;
}

llsa_status llsa_backward(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, const void *O,
                          const float *LSE, const int32_t *indices, const void *dO, void *dQ, void *dK, void *dV,
                          void *workspace, void *hip_stream) {
    if (!plan || !Q || !K || !V || !O || !LSE || !indices || !dO || !dQ || !dK || !dV || !workspace)
        return LLSA_ERR_NULL;
    if (any_misaligned16(Q, K, V, O, LSE, indices, dO, dQ, dK, dV) || misaligned(workspace, 256)) return LLSA_ERR_BAD_SHAPE;
    const Plan &p = plan->p;
    hipStream_t s = (hipStream_t)hip_stream;
    char *w = static_cast<char *>(workspace);
    const int call = g_timer.on ? g_timer.bwd_calls++ : 0;
    if (p.desc.bwd_repool) {
        StageScope sc(kPool, call, s);
        LLSA_TRY(launch_pool(p, Q, K, V, workspace, false, s));
    }
    float *D = reinterpret_cast<float *>(w + p.D_off);
    // Independent work goes to the plan's auxiliary stream, unless every stage is being timed one by one.
    std::lock_guard<std::mutex> lock(plan->aux.mu);
    Aux *aux = (g_timer.on && g_timer.filter < 0) ? nullptr : aux_for_call(plan, s);
    hipStream_t side = aux ? aux->side : s;
    if (!p.fast) {                                          // the MFMA dQ kernel produces D itself
        StageScope sc(kBwdPre, call, s);
        LLSA_TRY(launch_bwd_pre(p, O, dO, D, s));
    }
    // Alg. 2 needs only the indices, so it runs on the auxiliary stream beside kernels that do not read its
    // lists.  Where the coarse levels use the grouped kernels (they write per-query-block partials, need no list,
    // and a level above their range is dense and has none), that is behind dQ, in the shadow of those kernels:
    // they are bound by LDS and leave wave slots and registers free, which dQ does not.  Otherwise it is beside dQ.
    const bool shadow = aux && p.group;
    bool forked = false, joined = false;
    auto transpose = [&]() -> llsa_status {
        const int top_listed = p.Le < p.L ? p.Le : p.L - 1;    // highest level that has index lists in use
        if (aux) {
            LLSA_TRY(hipEventRecord(aux->ev[0], s));
            LLSA_TRY(hipStreamWaitEvent(side, aux->ev[0], 0));
            forked = true;
        }
        StageScope sc(kTranspose, call, side);              // bracketed on the stream it runs on
        LLSA_TRY(launch_csc(p, top_listed, indices, workspace, side));
        if (aux) {
            LLSA_TRY(hipEventRecord(aux->ev[1], side));
        }
        return LLSA_OK;
    };
    auto enqueue = [&]() -> llsa_status {
        if (!shadow) LLSA_TRY_ST(transpose());
        LevelTable t = make_level_table(p, K, V, indices, workspace);
        {
            StageScope sc(kDq, call, s);
            if (p.fast) LLSA_TRY(launch_dq_mfma(p, t, Q, O, dO, LSE, D, dQ, s));
            else LLSA_TRY(launch_dq_generic(p, t, Q, dO, LSE, D, dQ, s));
        }
        if (shadow) LLSA_TRY_ST(transpose());
        // the caller's stream waits for the key-major lists where it first reads them (which also joins the streams)
        hipEvent_t lists = aux ? aux->ev[1] : nullptr;
        if (lists && !shadow) {
            LLSA_TRY(hipStreamWaitEvent(s, lists, 0));
            joined = true;
        }
        // coarse levels first (fp32), fold them down level by level, then level 0 adds its parent's share
        {
            StageScope sc(kDkvCoarse, call, s);
            if (p.group) {                                  // levels above the grouped kernel's range first
                for (int l = p.Le; l > dkv_group_top(p); --l) LLSA_TRY(launch_dkv_mfma(p, t, l, Q, dO, LSE, D, workspace, dK, dV, s));
                LLSA_TRY(launch_dkv_group(p, t, Q, dO, LSE, D, workspace, s, shadow ? lists : nullptr, shadow ? side : nullptr,
                                          shadow ? aux->ev[2] : nullptr));
                if (shadow) joined = true;                  // the grouped launcher waits for the lists before its gathers
            } else for (int l = p.Le; l >= 1; --l) {
                if (p.fast) LLSA_TRY(launch_dkv_mfma(p, t, l, Q, dO, LSE, D, workspace, dK, dV, s));
                else LLSA_TRY(launch_dkv_generic(p, t, l, Q, dO, LSE, D, workspace, dK, dV, s));
            }
        }
        {
            StageScope sc(kUnpool, call, s);
            if (!p.fast)                                    // the MFMA path folds this into its slab reduction
                for (int l = p.Le; l >= 2; --l) LLSA_TRY(launch_unpool(p, l, workspace, s));
        }
        StageScope sc(kDkvFine, call, s);
        if (p.fast) LLSA_TRY(launch_dkv_mfma(p, t, 0, Q, dO, LSE, D, workspace, dK, dV, s));
        else LLSA_TRY(launch_dkv_generic(p, t, 0, Q, dO, LSE, D, workspace, dK, dV, s));
        return LLSA_OK;
    };
    const llsa_status st = enqueue();
    if (forked && !joined) {
        // A launch failed after the fork: still lead the auxiliary stream back into the caller's, so that a stream
        // capture in progress is not left with an unjoined branch.  Errors here cannot make the outcome worse.
        // (recorded again even if it was before: the side stream may have been given more work since)
        (void)hipEventRecord(aux->ev[1], side);
        (void)hipStreamWaitEvent(s, aux->ev[1], 0);
    }
    return st;
}

size_t llsa_kv_backward_mask_bytes(const llsa_plan_t *plan) {
    if (!plan) return 0;
    const size_t T = (size_t)plan->p.n[1];
    return ((size_t)plan->p.bh * T * T + 255) & ~(size_t)255;
}

llsa_status llsa_kv_backward_level0(const llsa_plan_t *plan, int32_t via_mask, const void *Q, const void *K, const void *V,
                                    const void *dO, const float *LSE, const int32_t *indices, void *mask,
                                    void *workspace, void *dK0, void *dV0, void *hip_stream) {
    if (!plan || !Q || !K || !V || !dO || !LSE || !indices || !workspace || !dK0 || !dV0 || (via_mask && !mask))
        return LLSA_ERR_NULL;
    if (any_misaligned16(Q, K, V, dO, LSE, indices, dK0, dV0, mask) || misaligned(workspace, 256)) return LLSA_ERR_BAD_SHAPE;
    const Plan &p = plan->p;
    if (!p.fast) return LLSA_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)hip_stream;
    char *w = static_cast<char *>(workspace);
    if (via_mask) LLSA_TRY(launch_mask_lists(p, indices, workspace, mask, s));
    else LLSA_TRY(launch_csc(p, 0, indices, workspace, s));
    LevelTable t = make_level_table(p, K, V, indices, workspace);
    LLSA_TRY(launch_dkv_mfma(p, t, 0, Q, dO, LSE, reinterpret_cast<const float *>(w + p.D_off), workspace, dK0, dV0, s, true));
    return LLSA_OK;
}

llsa_status llsa_reorder(int64_t batch_heads, int64_t N, int32_t d, int32_t dtype, int32_t inverse, const void *in,
                         void *out, void *hip_stream) {
    if (!in || !out) return LLSA_ERR_NULL;
    if (dtype != LLSA_F32 && dtype != LLSA_BF16) return LLSA_ERR_UNSUPPORTED;
    if (batch_heads < 1 || N < 1 || d < 1 || N > ((int64_t)1 << 30) || batch_heads > (1 << 20)) return LLSA_ERR_BAD_SHAPE;
    int bits = 0;
    while (((int64_t)1 << (2 * bits)) < N) ++bits;
    const int64_t row_bytes = (int64_t)d * (dtype == LLSA_F32 ? 4 : 2);
    if (((int64_t)1 << (2 * bits)) != N || row_bytes % 16 != 0 || row_bytes > (1 << 16)) return LLSA_ERR_BAD_SHAPE;
    const char *a = static_cast<const char *>(in), *b = static_cast<const char *>(out);
    const int64_t bytes = batch_heads * N * row_bytes;
    if (a < b + bytes && b < a + bytes) return LLSA_ERR_BAD_SHAPE;      // the copy is not in place
    LLSA_TRY(launch_reorder(batch_heads, N, (int)row_bytes, bits, inverse ? 1 : 0, in, out, (hipStream_t)hip_stream));
    return LLSA_OK;
}

llsa_status llsa_calibrate_mfma(float *out, int32_t iters, int32_t workgroups, void *hip_stream) {
    if (!out) return LLSA_ERR_NULL;
    if (iters < 1 || workgroups < 1 || workgroups > (1 << 20)) return LLSA_ERR_BAD_SHAPE;
    LLSA_TRY(launch_peak_mfma(out, iters, workgroups, (hipStream_t)hip_stream));
    return LLSA_OK;
}

llsa_status llsa_calibrate_copy(const void *src, void *dst, int64_t bytes, void *hip_stream) {
    if (!src || !dst) return LLSA_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0 || any_misaligned16(src, dst)) return LLSA_ERR_BAD_SHAPE;
    LLSA_TRY(launch_peak_copy(src, dst, bytes, (hipStream_t)hip_stream));
    return LLSA_OK;
}

int32_t llsa_stage_count(void) { return kStages; }

const char *llsa_stage_name(int32_t stage) { return (stage >= 0 && stage < kStages) ? kStageNames[stage] : ""; }

llsa_status llsa_stage_timing_begin(int32_t stage, int32_t max_calls) {
    StageTimer &t = g_timer;
    if (t.on || max_calls < 1 || max_calls > 4096 || stage >= kStages) return LLSA_ERR_BAD_SHAPE;
    const size_t n = (size_t)max_calls * kStages;
    t.ev.assign(2 * n, nullptr);
    t.rec.assign(n, 0);
    for (size_t i = 0; i < 2 * n; ++i)
        if (hipEventCreate(&t.ev[i]) != hipSuccess) {
            for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(t.ev[j]);
            t.ev.clear();
            return LLSA_ERR_RUNTIME;
        }
    t.filter = stage; t.max_calls = max_calls; t.fwd_calls = t.bwd_calls = 0; t.on = true;
    return LLSA_OK;
}

llsa_status llsa_stage_timing_end(double *ms_sum, int32_t *brackets) {
    StageTimer &t = g_timer;
    if (!t.on) return LLSA_ERR_BAD_SHAPE;
    if (!ms_sum || !brackets) return LLSA_ERR_NULL;
    llsa_status st = LLSA_OK;
    for (int i = 0; i < kStages; ++i) { ms_sum[i] = 0.0; brackets[i] = 0; }
    for (int c = 0; c < t.max_calls; ++c)
        for (int i = 0; i < kStages; ++i) {
            const size_t k = (size_t)c * kStages + i;
            if (t.rec[k] != 2) continue;
            float ms = 0.f;
            if (hipEventSynchronize(t.ev[2 * k + 1]) != hipSuccess ||
                hipEventElapsedTime(&ms, t.ev[2 * k], t.ev[2 * k + 1]) != hipSuccess) { st = LLSA_ERR_RUNTIME; continue; }
            ms_sum[i] += ms;
            brackets[i] += 1;
        }
    for (hipEvent_t e : t.ev) (void)hipEventDestroy(e);
    t.ev.clear(); t.rec.clear(); t.on = false;
    return st;
}

const char *llsa_status_string(llsa_status s) {
    switch (s) {
        case LLSA_OK: return "ok";
        case LLSA_ERR_NULL: return "null pointer";
        case LLSA_ERR_BAD_SHAPE: return "bad shape (N must be divisible by B^L; L >= 1; 0 <= Le <= L; K >= 1)";
        case LLSA_ERR_UNSUPPORTED: return "unsupported d / B / K / dtype / size";
        case LLSA_ERR_WORKSPACE: return "the problem's forward workspace exceeds the library's static one";
        case LLSA_ERR_RUNTIME: return "HIP launch failed";
    }
    return "unknown status";
}

}  // extern "C"
