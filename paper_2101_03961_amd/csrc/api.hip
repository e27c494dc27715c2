// C ABI of the Switch FFN library: argument checks, workspace layout, kernel
// sequencing, event-based kernel timing.  See include/switchffn.h.
#include <math.h>
#include <string.h>

#include <string>
#include <vector>

#include "common.h"

namespace sw {

int check_config(const switch_config *cfg) {
    if (!cfg) return SW_ERR_NULL;
    if (cfg->act_dtype != SW_F32 && cfg->act_dtype != SW_BF16) return SW_ERR_DTYPE;
    if (cfg->ffn_kind != SW_FFN_RELU && cfg->ffn_kind != SW_FFN_GEGLU) return SW_ERR_DTYPE;
    if (cfg->T < 0 || cfg->T >= (int64_t)1 << 31) return SW_ERR_SHAPE;
    if (cfg->n_groups < 0 || cfg->n_groups > 65536) return SW_ERR_SHAPE;
    if (cfg->n_groups > 1 && (cfg->T % cfg->n_groups) != 0) return SW_ERR_SHAPE;
    if (cfg->E < 1 || cfg->E > 4096) return SW_ERR_SHAPE;
    if (cfg->d_model < 1 || cfg->d_ff < 1) return SW_ERR_SHAPE;
    if (cfg->d_model >= (int64_t)1 << 24 || cfg->d_ff >= (int64_t)1 << 24) return SW_ERR_SHAPE;
    const int64_t mult = cfg->act_dtype == SW_BF16 ? 8 : 4;   // rows move as 16-byte chunks
    if (cfg->d_model % mult || cfg->d_ff % mult) return SW_ERR_SHAPE;
    if (!(cfg->capacity_factor > 0.0) || !isfinite(cfg->capacity_factor)) return SW_ERR_VALUE;
    if (!isfinite(cfg->alpha)) return SW_ERR_VALUE;
    if (!(cfg->expert_dropout >= 0.f && cfg->expert_dropout < 1.f)) return SW_ERR_VALUE;
    if (!(cfg->jitter_eps >= 0.f && cfg->jitter_eps < 1.f)) return SW_ERR_VALUE;
    if (cfg->ntlb_rounds < 0 || cfg->ntlb_rounds > 16) return SW_ERR_VALUE;
    if (cfg->flags & ~SW_FLAG_FUSED_DISPATCH) return SW_ERR_VALUE;
    // slot indices (expert * slots per expert + position) are kept in 32 bits
    const double n = cfg->n_groups > 1 ? (double)cfg->n_groups : 1.0;
    const double c = floor((double)cfg->T / n / (double)cfg->E * cfg->capacity_factor);
    if (c * n * (double)cfg->E >= 2147483647.0) return SW_ERR_SHAPE;
    if (cfg->act_dtype == SW_BF16) {
        // the bf16 GEMMs address one expert's matrices through 32-bit buffer descriptors
        const double f1 = (double)cfg->d_ff * (cfg->ffn_kind == SW_FFN_GEGLU ? 2.0 : 1.0);
        const double wide = (double)cfg->d_model > f1 ? (double)cfg->d_model : f1;
        if ((double)cfg->d_model * f1 * 2.0 >= 2147483647.0) return SW_ERR_SHAPE;
        if (c * n * wide * 2.0 >= 2147483647.0) return SW_ERR_SHAPE;
    }
    return SW_OK;
}

int64_t capacity_of(const switch_config *cfg) {
    const int64_t n = cfg->n_groups > 1 ? cfg->n_groups : 1;
    return (int64_t)floor((double)(cfg->T / n) / (double)cfg->E * cfg->capacity_factor);
}

Workspace layout_workspace(const switch_config *cfg) {
    Workspace w{};
    w.T = cfg->T; w.d = cfg->d_model; w.f = cfg->d_ff; w.E = cfg->E;
    w.geglu = cfg->ffn_kind == SW_FFN_GEGLU;
    w.f1 = w.geglu ? 2 * w.f : w.f;
    w.n = cfg->n_groups > 1 ? cfg->n_groups : 1;
    w.Tg = w.T / w.n;
    w.Cg = capacity_of(cfg);
    w.C = w.n * w.Cg;
    w.nbg = ceil_div(w.Tg, kRouteTB);
    w.nb = w.n * w.nbg;
    w.elt = cfg->act_dtype == SW_BF16 ? 2 : 4;
    w.nsplit = w.nb < 64 ? w.nb : 64;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t T = w.T, E = w.E, C = w.C, d = w.d, f = w.f, f1 = w.f1, nb = w.nb;
    w.probs = take(T * E * 4);
    w.idx = take(T * 4);
    w.gate = take(T * 4);
    w.local_rank = take(nb * kRouteTB * 4);
    w.block_counts = take(nb * E * 4);
    w.block_psum = take(nb * E * 4);
    w.block_off = take(nb * E * 4);
    w.counts = take(E * 4);
    w.counts_g = take((size_t)w.n * E * 4);
    w.psum_g = take((size_t)w.n * E * 4);
    w.grp_off = take((size_t)w.n * E * 4);
    w.loss_part = take(8 * 8);
    w.kept = take(E * 4);
    // 128 entries of padding: the GEMMs that gather k-rows read the table a step past an
    // expert's last slot (and mask what they read)
    w.slot_token = take((E * C + 128) * 4);
    w.slot_gate = take(E * C * 4);
    w.slot_off = take((E * C + 128) * 4);
    // dispatch and combine inside the GEMMs: bf16, and x / dy / y addressed through one buffer
    // descriptor with 32-bit byte offsets
    w.fused = cfg->act_dtype == SW_BF16 && (cfg->flags & SW_FLAG_FUSED_DISPATCH) &&
              (double)T * (double)d * 2.0 < 2147483647.0;
    w.tok_slot = take(T * 4);
    w.Xd = take(E * C * d * w.elt);
    w.H = take(w.geglu ? E * C * f1 * w.elt : 0);
    w.A = take(E * C * f * w.elt);
    w.O = take(E * C * d * w.elt);
    w.dO = take(E * C * d * w.elt);
    w.dA = take(w.geglu ? E * C * f * w.elt : 0);
    w.dH = take(E * C * f1 * w.elt);
    w.dXd = take(E * C * d * w.elt);
    w.dgate = take(T * 4);
    w.dlogits = take(T * E * 4);
    w.dWr_part = take((size_t)w.nsplit * d * E * 4);
    w.dbr_part = take((size_t)ceil_div(w.T, kRouteTB) * E * 4);
    w.dpad = ceil_div(w.d, 32) * 32;
    // noise parameters first: the router's layout depends on the jitter
    Noise &nz = w.noise;
    const uint32_t seed_hi = (uint32_t)(cfg->seed >> 32);
    nz.seed_lo = (uint32_t)cfg->seed;
    nz.jitter_term = seed_hi + 1u * 0x7F4A7C15u;
    nz.dropout_term = seed_hi + 2u * 0x7F4A7C15u;
    nz.dropout = cfg->expert_dropout > 0.f;
    nz.jitter = cfg->jitter_eps > 0.f;
    nz.drop_thr = (uint32_t)floor((double)cfg->expert_dropout * 65536.0);
    nz.drop_scale = (float)(65536.0 / (65536.0 - (double)nz.drop_thr));
    nz.jitter_eps = cfg->jitter_eps;
    const bool jit_mfma = nz.jitter && cfg->act_dtype == SW_BF16;
    w.dpad_r = jit_mfma ? 3 * w.dpad : w.dpad;
    w.etiles = ceil_div(w.E, 128);
    w.wsplit = take((size_t)w.etiles * 3 * 128 * w.dpad_r * 2);
    w.wsplit_b = take((size_t)w.etiles * d * 256 * 2);
    w.dl_split = take((size_t)w.etiles * T * 256 * 2);
    w.xj = take(jit_mfma ? T * (size_t)w.dpad_r * 2 : 0);
    w.no_slot = take(jit_mfma ? T * 4 : 0);
    w.tps_m = ceil_div(ceil_div(w.T, 85), 64) * 64;
    if (w.tps_m < 64) w.tps_m = 64;   // empty batch
    w.nsplit_m = ceil_div(w.T, w.tps_m);
    w.dWr_part_m = take((size_t)w.etiles * w.nsplit_m * (jit_mfma ? 2 * (size_t)w.dpad : d) * 256 * 4);
    w.relu_bits = take(E * ceil_div(f, kGemmTile) * ceil_div(C, kGemmTile) * kReluBitsPerTile);
    w.ntlb_rounds = cfg->ntlb_rounds;
    if (w.ntlb_rounds > 0) {
        const size_t nE = (size_t)w.n * E * 4;
        w.ntlb_logits = take(T * E * 4);
        w.ntlb_asked = take(T * 4);
        w.ntlb_cnt = take(nE);
        w.ntlb_used = take(nE);
        w.ntlb_free = take(nE);
        w.ntlb_base = take(nE);
    }
    w.total = off;
    return w;
}

// ---- event-based kernel timing -------------------------------------------------
struct ProfEntry {
    const char *name;
    double total_ms;
    int64_t launches;
};
struct ProfRecord {
    int entry;
    hipEvent_t start, stop;
};
static bool g_prof_on = false;
static std::vector<ProfEntry> g_entries;
static std::vector<ProfRecord> g_records;     // pending (not yet collected)
static std::vector<hipEvent_t> g_event_pool;  // free events
static int g_open = -1;

static hipEvent_t get_event() {
    if (!g_event_pool.empty()) {
        hipEvent_t e = g_event_pool.back();
        g_event_pool.pop_back();
        return e;
    }
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void prof_begin(const char *name, hipStream_t s) {
    if (!g_prof_on) return;
    int entry = -1;
    for (size_t i = 0; i < g_entries.size(); ++i)
        if (strcmp(g_entries[i].name, name) == 0) { entry = (int)i; break; }
    if (entry < 0) {
        g_entries.push_back({name, 0.0, 0});
        entry = (int)g_entries.size() - 1;
    }
    ProfRecord r{entry, get_event(), get_event()};
    if (!r.start || !r.stop) return;
    (void)hipEventRecord(r.start, s);
    g_records.push_back(r);
    g_open = (int)g_records.size() - 1;
}

void prof_end(hipStream_t s) {
    if (!g_prof_on || g_open < 0) return;
    (void)hipEventRecord(g_records[g_open].stop, s);
    g_open = -1;
}

static int status_of(hipError_t e) { return e == hipSuccess ? SW_OK : SW_ERR_LAUNCH; }

static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace sw

// ---- library-owned scratch for callers that cannot allocate --------------------
// One copy per GPU (device memory of the loaded code object, held until the process ends).
// In host code the array's name is only a handle: the device address is asked for once per
// device, with that device current, and only that address is ever passed on.
static __device__ __align__(256) unsigned char scratch[SW_STATIC_SCRATCH_BYTES];

namespace sw {
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mu;

// device address of `scratch` on the current device
static int static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SW_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SW_ERR_LAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SW_OK;
}
}  // namespace sw

using namespace sw;

extern "C" {

int switch_capacity(const switch_config *cfg, int64_t *capacity_out) {
    if (!cfg || !capacity_out) return SW_ERR_NULL;
    int st = check_config(cfg);
    if (st != SW_OK) return st;
    *capacity_out = capacity_of(cfg);
    return SW_OK;
}

int switch_workspace_size(const switch_config *cfg, size_t *bytes_out) {
    if (!cfg || !bytes_out) return SW_ERR_NULL;
    int st = check_config(cfg);
    if (st != SW_OK) return st;
    *bytes_out = layout_workspace(cfg).total;
    return SW_OK;
}

// 4-byte words set to zero (stays valid under stream capture, unlike a memset node)
__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t *__restrict__ p, size_t words) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += stride) p[i] = 0u;
}

static int fill_zero(void *p, size_t bytes, hipStream_t s) {
    const size_t words = bytes / 4;
    if (words == 0) return SW_OK;
    size_t blocks = (words + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint32_t *)p, words);
    return status_of(hipGetLastError());
}

// The forward pass on a workspace that has been checked: argument checks, then launches only.
static int forward_on(const switch_config *cfg, const Workspace &w, const void *x, const float *W_r,
                      const float *b_r, const void *W_in, const void *W_out, void *y,
                      int32_t *expert_index, float *gate, int32_t *position_in_expert,
                      uint8_t *dropped, int32_t *expert_counts, float *aux_loss,
                      float *router_logits, char *ws, hipStream_t s) {
    int st;
    const int dt = cfg->act_dtype;
    auto gemm = dt == SW_BF16 ? launch_gemm_bf16 : launch_gemm_f32;
    // the re-routing stages rank the experts by logit: keep the logits if the caller does not
    if (w.ntlb_rounds > 0 && !router_logits) router_logits = (float *)(ws + w.ntlb_logits);

    if (router_fwd_mfma_supported(w, dt))
        st = status_of(launch_router_fwd_mfma(w, x, W_r, b_r, ws, expert_index, gate,
                                              router_logits, s));
    else
        st = status_of(launch_router_fwd(w, dt, x, W_r, b_r, ws, expert_index, gate,
                                         router_logits, s));
    if (st) return st;
    if ((st = status_of(launch_route_scan(w, ws, expert_counts, s)))) return st;
    if ((st = status_of(launch_dispatch(w, dt, cfg->alpha, x, ws, position_in_expert, dropped,
                                        aux_loss, router_logits, expert_index, gate, y, s))))
        return st;
    const TokenMajor tm{x, nullptr, y};
    // fused: rows of tokens without a slot are +0 (cleared above, or here once the re-routing
    // stages have run), all others are written by the second GEMM
    if (w.fused && !zero_rows_with_positions(w) &&
        (st = status_of(launch_zero_dropped(w, ws, y, s))))
        return st;
    if ((st = status_of(gemm(GEMM_FWD1, w, ws, W_in, W_out, nullptr, nullptr, tm, s)))) return st;
    if (w.geglu && (st = status_of(launch_geglu_fwd(w, dt, ws, s)))) return st;
    if ((st = status_of(gemm(GEMM_FWD2, w, ws, W_in, W_out, nullptr, nullptr, tm, s)))) return st;
    if (!w.fused && (st = status_of(launch_combine(w, dt, ws, y, s)))) return st;
    return SW_OK;
}

// pointer checks of the forward pass (T > 0)
static int check_forward_pointers(const void *x, const float *W_r, const float *b_r,
                                  const void *W_in, const void *W_out, void *y,
                                  int32_t *expert_index, float *gate, int32_t *position_in_expert,
                                  uint8_t *dropped, int32_t *expert_counts, float *aux_loss,
                                  float *router_logits) {
    if (!x || !W_r || !W_in || !W_out || !y || !expert_index || !gate || !position_in_expert ||
        !dropped || !expert_counts || !aux_loss)
        return SW_ERR_NULL;
    if (!aligned16(x) || !aligned16(W_r) || !aligned16(W_in) || !aligned16(W_out) ||
        !aligned16(y) || (b_r && !aligned16(b_r)) || (router_logits && !aligned16(router_logits)))
        return SW_ERR_ALIGN;
    return SW_OK;
}

int switch_forward(const switch_config *cfg, const void *x, const float *W_r, const float *b_r,
                   const void *W_in, const void *W_out, void *y, int32_t *expert_index,
                   float *gate, int32_t *position_in_expert, uint8_t *dropped,
                   int32_t *expert_counts, float *aux_loss, float *router_logits, void *workspace,
                   size_t workspace_bytes, void *hip_stream) {
    int st = check_config(cfg);
    if (st != SW_OK) return st;
    hipStream_t s = (hipStream_t)hip_stream;
    if (cfg->T == 0) {   // empty batch: no token, no routing; counts and loss are zero
        if (!expert_counts || !aux_loss) return SW_ERR_NULL;
        if ((st = fill_zero(expert_counts, (size_t)cfg->E * 4, s))) return st;
        return fill_zero(aux_loss, 4, s);
    }
    if ((st = check_forward_pointers(x, W_r, b_r, W_in, W_out, y, expert_index, gate,
                                     position_in_expert, dropped, expert_counts, aux_loss,
                                     router_logits)))
        return st;
    const Workspace w = layout_workspace(cfg);
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < w.total)
        return SW_ERR_WORKSPACE;
    return forward_on(cfg, w, x, W_r, b_r, W_in, W_out, y, expert_index, gate, position_in_expert,
                      dropped, expert_counts, aux_loss, router_logits, (char *)workspace, s);
}

int switch_forward_static(const switch_config *cfg, const void *x, const float *W_r,
                          const float *b_r, const void *W_in, const void *W_out, void *y,
                          int32_t *expert_index, float *gate, int32_t *position_in_expert,
                          uint8_t *dropped, int32_t *expert_counts, float *aux_loss,
                          float *router_logits, void *hip_stream) {
    int st = check_config(cfg);
    if (st != SW_OK) return st;
    // the size limit comes first: it depends on the configuration alone
    const Workspace w = layout_workspace(cfg);
    if (w.total > (size_t)SW_STATIC_SCRATCH_BYTES) return SW_ERR_STATIC_LIMIT;
    hipStream_t s = (hipStream_t)hip_stream;
    if (cfg->T == 0) {
        if (!expert_counts || !aux_loss) return SW_ERR_NULL;
        if ((st = fill_zero(expert_counts, (size_t)cfg->E * 4, s))) return st;
        return fill_zero(aux_loss, 4, s);
    }
    if ((st = check_forward_pointers(x, W_r, b_r, W_in, W_out, y, expert_index, gate,
                                     position_in_expert, dropped, expert_counts, aux_loss,
                                     router_logits)))
        return st;
    void *ws = nullptr;
    if ((st = static_scratch(&ws))) return st;
    // Nothing in the forward pass reads a workspace word before a kernel of the same call has
    // written it, so what an earlier call left in the array needs no clearing.
    return forward_on(cfg, w, x, W_r, b_r, W_in, W_out, y, expert_index, gate, position_in_expert,
                      dropped, expert_counts, aux_loss, router_logits, (char *)ws, s);
}

int switch_backward(const switch_config *cfg, const void *dy, float d_aux, const void *x,
                    const float *W_r, const float *b_r, const void *W_in, const void *W_out,
                    void *dx, float *dW_r, float *db_r, void *dW_in, void *dW_out, void *workspace,
                    size_t workspace_bytes, void *hip_stream) {
    (void)b_r;   // the bias enters the gradients only through the saved probabilities
    int st = check_config(cfg);
    if (st != SW_OK) return st;
    if (!isfinite(d_aux)) return SW_ERR_VALUE;
    if (cfg->T == 0) {   // empty batch: every weight gradient is an empty sum
        if (!dW_r || !dW_in || !dW_out) return SW_ERR_NULL;
        if (!aligned16(dW_r) || !aligned16(dW_in) || !aligned16(dW_out)) return SW_ERR_ALIGN;
        hipStream_t s0 = (hipStream_t)hip_stream;
        const size_t elt = cfg->act_dtype == SW_BF16 ? 2 : 4;
        const size_t wbytes = (size_t)cfg->E * cfg->d_model * cfg->d_ff * elt;
        const size_t in_mult = cfg->ffn_kind == SW_FFN_GEGLU ? 2 : 1;
        if ((st = fill_zero(dW_r, (size_t)cfg->d_model * cfg->E * 4, s0))) return st;
        if (db_r && (st = fill_zero(db_r, (size_t)cfg->E * 4, s0))) return st;
        if ((st = fill_zero(dW_in, wbytes * in_mult, s0))) return st;
        return fill_zero(dW_out, wbytes, s0);
    }
    if (!dy || !x || !W_r || !W_in || !W_out || !dx || !dW_r || !dW_in || !dW_out)
        return SW_ERR_NULL;
    if (!aligned16(dy) || !aligned16(x) || !aligned16(W_r) || !aligned16(W_in) ||
        !aligned16(W_out) || !aligned16(dx) || !aligned16(dW_r) || !aligned16(dW_in) ||
        !aligned16(dW_out) || (db_r && !aligned16(db_r)))
        return SW_ERR_ALIGN;
    const Workspace w = layout_workspace(cfg);
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < w.total)
        return SW_ERR_WORKSPACE;
    char *ws = (char *)workspace;
    hipStream_t s = (hipStream_t)hip_stream;
    const int dt = cfg->act_dtype;
    auto gemm = dt == SW_BF16 ? launch_gemm_bf16 : launch_gemm_f32;

    const TokenMajor tm{x, dy, nullptr};
    // fused: only the gate gradient is left of the combine's backward pass (dy is read by the
    // GEMMs through the slot -> token table)
    if (w.fused)
        st = status_of(launch_gate_grad(w, dy, ws, s));
    else
        st = status_of(launch_combine_bwd(w, dt, dy, ws, s));
    if (st) return st;
    if ((st = status_of(gemm(GEMM_DGRAD2, w, ws, W_in, W_out, dW_in, dW_out, tm, s)))) return st;
    if (w.geglu && (st = status_of(launch_geglu_bwd(w, dt, ws, s)))) return st;
    // dH is consumed right after it is produced (the first-layer data gradient walks the
    // experts backwards, see launch_gemm_bf16), then the two weight gradients
    if ((st = status_of(gemm(GEMM_DGRAD1, w, ws, W_in, W_out, dW_in, dW_out, tm, s)))) return st;
    if ((st = status_of(gemm(GEMM_WGRAD1, w, ws, W_in, W_out, dW_in, dW_out, tm, s)))) return st;
    if ((st = status_of(gemm(GEMM_WGRAD2, w, ws, W_in, W_out, dW_in, dW_out, tm, s)))) return st;
    if ((st = status_of(launch_router_bwd(w, dt, cfg->alpha, d_aux, x, W_r, ws, dx, dW_r, db_r, s))))
        return st;
    return SW_OK;
}

const char *switch_status_string(int status) {
    switch (status) {
    case SW_OK: return "ok";
    case SW_ERR_NULL: return "a required pointer is NULL";
    case SW_ERR_SHAPE: return "shape out of range (T, E, d_model, d_ff; 16-byte row chunks)";
    case SW_ERR_VALUE:
        return "capacity_factor must be finite and > 0; alpha, d_aux finite; expert_dropout and "
               "jitter_eps in [0, 1); ntlb_rounds in 0..16; flags: known bits only";
    case SW_ERR_DTYPE: return "act_dtype must be SW_F32 or SW_BF16, ffn_kind SW_FFN_RELU or SW_FFN_GEGLU";
    case SW_ERR_WORKSPACE: return "workspace NULL, not 256-byte aligned, or too small";
    case SW_ERR_ALIGN: return "tensor pointer not 16-byte aligned";
    case SW_ERR_LAUNCH: return "HIP launch failed";
    case SW_ERR_STATE: return "profiling call out of order";
    case SW_ERR_STATIC_LIMIT:
        return "configuration needs more workspace than the library's static scratch "
               "(SW_STATIC_SCRATCH_BYTES); use switch_forward with a caller workspace";
    default: return "unknown status";
    }
}

int switch_profile_enable(int on) {
    if (on) {
        for (auto &r : g_records) {
            g_event_pool.push_back(r.start);
            g_event_pool.push_back(r.stop);
        }
        g_records.clear();
        g_entries.clear();
        g_open = -1;
    }
    g_prof_on = on != 0;
    return SW_OK;
}

int switch_profile_collect(void) {
    if (g_open >= 0) return SW_ERR_STATE;
    for (auto &r : g_records) {
        if (hipEventSynchronize(r.stop) != hipSuccess) return SW_ERR_LAUNCH;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) return SW_ERR_LAUNCH;
        g_entries[r.entry].total_ms += ms;
        g_entries[r.entry].launches += 1;
        g_event_pool.push_back(r.start);
        g_event_pool.push_back(r.stop);
    }
    g_records.clear();
    return SW_OK;
}

int switch_profile_count(void) { return (int)g_entries.size(); }

int switch_profile_get(int i, const char **name, double *total_ms, int64_t *launches) {
    if (i < 0 || i >= (int)g_entries.size()) return SW_ERR_SHAPE;
    if (name) *name = g_entries[i].name;
    if (total_ms) *total_ms = g_entries[i].total_ms;
    if (launches) *launches = g_entries[i].launches;
    return SW_OK;
}

}  // extern "C"
