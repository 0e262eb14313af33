// C ABI of libconfu_verify.so: argument checks on host scalars, launch planning, dispatch.
#include <atomic>
#include <cstring>

#include "tv_internal.hpp"

namespace tv {

namespace {

int device_cu_count() {
    static std::atomic<int> cached{0};
    int n = cached.load(std::memory_order_relaxed);
    if (n > 0) return n;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
        prop.multiProcessorCount > 0)
        n = prop.multiProcessorCount;
    else
        n = 256;      // MI355X
    cached.store(n, std::memory_order_relaxed);
    return n;
}

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

int check_attn_desc(const tv_attn_desc* d) {
    if (!d || d->struct_size != sizeof(tv_attn_desc)) return TV_ERR_INVALID_ARG;
    if (d->B < 1 || d->B > 65535 || d->M < 1 || d->M > TV_MAX_ROWS || d->Hq < 1 || d->Hkv < 1 || d->Hq % d->Hkv != 0)
        return TV_ERR_INVALID_ARG;      // (a grid dimension counts the sequences)
    if (d->Hq / d->Hkv > 16) return TV_ERR_INVALID_ARG;
    if (d->soft_len < 0 || d->max_prefix_len < d->soft_len || d->num_splits < 0) return TV_ERR_INVALID_ARG;
    if (d->wg_row_blocks != 0 && d->wg_row_blocks != 1 && d->wg_row_blocks != 2 && d->wg_row_blocks != 4)
        return TV_ERR_INVALID_ARG;
    if (d->sum_prefix_len < 0 || d->sum_prefix_len > (int64_t)d->B * d->max_prefix_len) return TV_ERR_INVALID_ARG;
    if (!(d->softmax_scale > 0.f)) return TV_ERR_INVALID_ARG;
    if (d->kv_token_stride < 0 || d->kv_head_stride < 0) return TV_ERR_INVALID_ARG;
    if (d->dtype == TV_DTYPE_F32) {
        if (d->D != 64 && d->D != 128) return TV_ERR_UNSUPPORTED;
    } else if (d->dtype == TV_DTYPE_BF16) {
        if (d->D != 128) return TV_ERR_UNSUPPORTED;
    } else {
        return TV_ERR_INVALID_ARG;
    }
    const int64_t hs = d->kv_head_stride ? d->kv_head_stride : d->D;
    const int64_t ts = d->kv_token_stride ? d->kv_token_stride : (int64_t)d->Hkv * d->D;
    const int vec = (d->dtype == TV_DTYPE_F32) ? 4 : 8;      // 16-byte loads
    if (hs < d->D || ts < d->D || hs % vec != 0 || ts % vec != 0) return TV_ERR_INVALID_ARG;   // token-major and head-major pools both fit
    // byte offsets inside one sequence are formed in 32 bits
    const int elem = (d->dtype == TV_DTYPE_F32) ? 4 : 2;
    if (((int64_t)d->max_prefix_len + d->M) * ts * elem >= ((int64_t)1 << 32)) return TV_ERR_INVALID_ARG;
    return TV_OK;
}

}  // namespace

static int plan_attention_uncached(const tv_attn_desc& d, AttnPlan* plan);

// The plan depends on the descriptor (and the device's CU count) only, and a serving loop hands over the same
// descriptor layer after layer: each thread remembers the last one it planned (a few microseconds of host time per
// call otherwise).  The descriptor is compared field by field as bytes; its padding-free layout makes that exact.
int plan_attention(const tv_attn_desc& d, AttnPlan* plan) {
    static_assert(sizeof(tv_attn_desc) == 72, "byte-wise comparison assumes a layout without padding");
    struct Last { tv_attn_desc d; AttnPlan p; int rc; int cus; bool valid; };
    thread_local Last last{};
    const int cus = device_cu_count();
    if (last.valid && last.cus == cus && std::memcmp(&last.d, &d, sizeof d) == 0) {
        *plan = last.p;
        return last.rc;
    }
    AttnPlan p{};
    const int rc = plan_attention_uncached(d, &p);
    last.d = d; last.p = p; last.rc = rc; last.cus = cus; last.valid = true;
    *plan = p;
    return rc;
}

static int plan_attention_uncached(const tv_attn_desc& d, AttnPlan* plan) {
    AttnPlan p{};
    p.G = d.Hq / d.Hkv;
    if (d.dtype == TV_DTYPE_F32) {
        p.row_blocks = (d.M + 15) / 16;
        p.n_chunks = 1;
        p.total_bytes = 0;
        *plan = p;
        return TV_OK;
    }
    const int rows = p.G * d.M;
    const int rb_needed = (rows + 63) / 64;
    const int n_tiles = (d.max_prefix_len + d.M + 31) / 32;
    // Workgroup shape (rb 64-row blocks per workgroup, 4/rb key streams) and number of key ranges n: what the
    // caller fixes is taken as given, the rest is chosen by a small cost model of the kernel, in microseconds,
    // fitted to measurements on MI355X (one and four sequences, 1k .. 64k cached tokens each, all three shapes,
    // pools larger than the last-level cache).  A workgroup takes
    //   t = fixed(rb) + rounds * per_round(rb)
    // with rounds = tiles of its longest key stream, fixed = launch, prologue and epilogue (larger shapes merge
    // and store more rows), per_round = one 32-key tile per stream (a little more on long runs, where the clock
    // settles lower); one workgroup runs per CU at a time; the second kernel adds 3.3 when n > 1.
    // The lengths are on the device, so the model prices two batches: every sequence at max_prefix_len
    // (all workgroups alike: whole waves of them, waves * t), and a ragged one whose lengths average 0.55 of the
    // longest, which is near max_prefix_len (U{512..8192} has that mean; see t_ragged below).  The choice is the candidate
    // whose worse regret over the two is smallest; one sequence has only the first case.  With the caller's
    // sum_prefix_len the batch is known instead: equal lengths when the mean is within a tenth of the maximum,
    // else the ragged model with that mean.
    const int cus = device_cu_count();
    const int max_n = n_tiles / 8 > 1 ? (n_tiles / 8 < 64 ? n_tiles / 8 : 64) : 1;     // at least eight tiles per range
    const bool mean_known = d.B > 1 && d.sum_prefix_len > 0 && d.max_prefix_len > 0;
    const double known_mean = mean_known ? (double)d.sum_prefix_len / ((double)d.B * d.max_prefix_len) : 1.0;
    const double ragged_mean = mean_known ? known_mean : 0.55;
    auto model_us = [&](int rb, int n, double* t_uniform, double* t_ragged) {
        const int streams = 4 / rb;
        const int64_t wgs = (int64_t)d.B * d.Hkv * ((rb_needed + rb - 1) / rb) * n;
        const int64_t waves = (wgs + cus - 1) / cus;
        const int rounds = (n_tiles + n * streams - 1) / (n * streams);
        // (64-row workgroups that all run at once - no more of them than CUs - start and step faster than when a
        //  second wave of them follows: 5.2 + r * 1.5..1.68 against 6.5 + r * 1.6..1.85, both measured)
        const bool at_once = wgs <= cus;
        const double fixed = rb == 1 ? (at_once ? 5.2 : 6.5) : rb == 2 ? 11.6 : 15.5;
        auto per_round = [&](double r) {
            if (rb == 1 && at_once) return 1.50 + 0.18 * (r <= 5 ? 0.0 : r >= 9 ? 1.0 : (r - 5) / 4.0);
            if (rb == 1) return 1.60 + 0.25 * (r <= 17 ? 0.0 : r >= 33 ? 1.0 : (r - 17) / 16.0);
            if (rb == 2) return 1.12 + 0.30 * (r <= 9 ? 0.0 : r >= 17 ? 1.0 : (r - 9) / 8.0);
            return 1.35 + 0.08 * (r <= 9 ? 0.0 : r >= 33 ? 1.0 : (r - 9) / 24.0);
        };
        auto wg_us = [&](double r) { return fixed + r * per_round(r); };
        const double combine = n > 1 ? 3.3 : 0.0;
        *t_uniform = (double)waves * wg_us(rounds) + combine;
        // Ragged: workgroup times spread evenly from the longest sequence's down to the shortest's (lengths uniform
        // on [2*mean - 1, 1] of the maximum), dispatched longest first.  The last workgroup ends no earlier than the
        // longest one, than the sum over all CUs, and - with more workgroups than CUs - than a second workgroup
        // started when the shortest of the first wave has finished.
        const double w = (double)wgs / cus;
        const double shortest = ragged_mean > 0.5 ? 2.0 * ragged_mean - 1.0 : 0.0;
        const double t_max = wg_us(rounds), t_mean = wg_us(ragged_mean * rounds), t_min = wg_us(shortest * rounds);
        double t = t_max > w * t_mean ? t_max : w * t_mean;
        if (w > 1.0 && w <= 2.0) {
            const double two = 2.0 * (t_max - (t_max - t_min) / w);
            if (two > t) t = two;
        } else if (w > 2.0) {
            const double more = w * t_mean + 0.5 * t_min;
            if (more > t) t = more;
        }
        *t_ragged = t + combine;
    };
    auto allowed = [&](int rb, int n) {
        if (d.wg_row_blocks ? rb != d.wg_row_blocks : (rb_needed % rb != 0)) return false;
        if (d.num_splits > 0) return n == (d.num_splits < max_n ? d.num_splits : max_n);
        return n <= max_n;
    };
    int best_rb = 0, best_n = 0;
    {
        double min_u = 1e30, min_r = 1e30;
        for (int rb = 1; rb <= 4; rb *= 2)
            for (int n = 1; n <= 64; ++n) {
                if (!allowed(rb, n)) continue;
                double tu, tr;
                model_us(rb, n, &tu, &tr);
                if (tu < min_u) min_u = tu;
                if (tr < min_r) min_r = tr;
            }
        double best_regret = 1e30, best_u = 1e30;
        for (int rb = 1; rb <= 4; rb *= 2)
            for (int n = 1; n <= 64; ++n) {
                if (!allowed(rb, n)) continue;
                double tu, tr;
                model_us(rb, n, &tu, &tr);
                const double ru = tu - min_u, rr = tr - min_r;
                double regret;
                if (d.B == 1 || (mean_known && known_mean >= 0.9)) regret = ru;       // equal lengths
                else if (mean_known) regret = rr;                                     // ragged, mean known
                else regret = ru > rr ? ru : rr;
                // (ties: the smaller time for equal lengths, then more ranges - the same rounds for the longest stream,
                //  fewer for the others)
                if (regret < best_regret || (regret == best_regret && (tu < best_u || (tu == best_u && n > best_n)))) {
                    best_regret = regret; best_u = tu; best_rb = rb; best_n = n;
                }
            }
    }
    if (best_rb == 0) return TV_ERR_INVALID_ARG;
    p.rb_per_wg = best_rb;
    p.row_blocks = (rb_needed + p.rb_per_wg - 1) / p.rb_per_wg * p.rb_per_wg;
    const int n = best_n;
    p.n_chunks = n;
    if (n > 1) {
        const size_t blocks = (size_t)d.B * d.Hkv * p.row_blocks * n;
        p.part_o_bytes = up256(blocks * 64 * 128 * 2);       // bf16
        p.part_ml_bytes = up256(blocks * 64 * 2 * sizeof(float));
    }
    p.total_bytes = p.part_o_bytes + p.part_ml_bytes;
    *plan = p;
    return TV_OK;
}

}  // namespace tv

using namespace tv;

extern "C" {

int tv_version(void) { return 210; }

static std::atomic<int> g_wait_limit{0};

int tv_set_wait_limit(int polls) { return g_wait_limit.exchange(polls < 0 ? 0 : polls); }

const char* tv_error_string(int code) {
    switch (code) {
        case TV_OK: return "ok";
        case TV_ERR_INVALID_ARG: return "invalid argument";
        case TV_ERR_WORKSPACE: return "workspace missing or too small";
        case TV_ERR_LAUNCH: return "HIP launch error";
        case TV_ERR_UNSUPPORTED: return "unsupported head dimension or dtype";
        default: return code < 0 ? "malformed tree" : "unknown error";
    }
}

int tv_build_mask_host(const int32_t* parent, const uint8_t* kind, int M, uint64_t* bits) {
    if (!parent || !kind || M < 1 || M > TV_MAX_ROWS) return TV_ERR_INVALID_ARG;
    int bad = 0;
    for (int i = 0; i < M; ++i) {
        const int p = parent[i];
        if (p < -1 || p >= i) bad |= TV_STATUS_BAD_PARENT;
        if (kind[i] != TV_KIND_NODE && kind[i] != TV_KIND_CONTEMPLATE) bad |= TV_STATUS_BAD_KIND;
        else if (p >= 0 && p < i && kind[i] == TV_KIND_NODE && kind[p] == TV_KIND_CONTEMPLATE)
            bad |= TV_STATUS_BAD_KIND;
    }
    if (bad) return -bad;
    if (bits) {
        for (int i = 0; i < M; ++i) {
            uint64_t w[2] = {0, 0};
            for (int j = i; j >= 0; j = parent[j]) w[j >> 6] |= (uint64_t)1 << (j & 63);
            bits[2 * i] = w[0];
            bits[2 * i + 1] = w[1];
        }
    }
    return TV_OK;
}

int tv_attention_workspace_bytes(const tv_attn_desc* desc, size_t* out_bytes) {
    if (!out_bytes) return TV_ERR_INVALID_ARG;
    const int rc = check_attn_desc(desc);
    if (rc != TV_OK) return rc;
    AttnPlan p;
    const int prc = plan_attention(*desc, &p);
    if (prc != TV_OK) return prc;
    *out_bytes = p.total_bytes;
    return TV_OK;
}

int tv_attention_plan(const tv_attn_desc* desc, int32_t* wg_row_blocks, int32_t* key_ranges) {
    if (!wg_row_blocks || !key_ranges) return TV_ERR_INVALID_ARG;
    const int rc = check_attn_desc(desc);
    if (rc != TV_OK) return rc;
    AttnPlan p;
    const int prc = plan_attention(*desc, &p);
    if (prc != TV_OK) return prc;
    *wg_row_blocks = desc->dtype == TV_DTYPE_BF16 ? p.rb_per_wg : 1;
    *key_ranges = p.n_chunks;
    return TV_OK;
}

int tv_prepare_tree(int32_t B, int32_t M, const int32_t* parent, const uint8_t* kind, void* prepared,
                    size_t prepared_bytes, void* hip_stream) {
    if (B < 1 || B > 65535 || M < 1 || M > TV_MAX_ROWS || !parent || !kind || !prepared) return TV_ERR_INVALID_ARG;
    if (((uintptr_t)prepared & 15) || prepared_bytes < (size_t)B * TV_PREPARED_TREE_BYTES) return TV_ERR_INVALID_ARG;
    const hipError_t e = launch_prepare_tree(parent, kind, B, M, static_cast<PreparedTree*>(prepared),
                                             static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TV_OK : TV_ERR_LAUNCH;
}

// Checks, plan and launch shared by the two attention entry points.
static int enqueue_attention(const tv_attn_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                             const int64_t* kv_offset, const int32_t* prefix_len, const int32_t* parent,
                             const uint8_t* kind, const void* prepared_tree, void* out, float* lse, int32_t* status,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    const int rc = check_attn_desc(desc);
    if (rc != TV_OK) return rc;
    if (!q || !k_pool || !v_pool || !kv_offset || !prefix_len || !parent || !kind || !out || !status)
        return TV_ERR_INVALID_ARG;
    const uintptr_t align_or = (uintptr_t)q | (uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)out | (uintptr_t)prepared_tree;
    if (align_or & 15) return TV_ERR_INVALID_ARG;
    AttnPlan p;
    const int prc = plan_attention(*desc, &p);
    if (prc != TV_OK) return prc;
    if (p.total_bytes > 0) {
        if (!workspace || workspace_bytes < p.total_bytes || ((uintptr_t)workspace & 255)) return TV_ERR_WORKSPACE;
    }
    AttnArgs a{};
    a.q = q; a.k = k_pool; a.v = v_pool;
    a.kv_offset = kv_offset; a.prefix_len = prefix_len; a.parent = parent; a.kind = kind;
    a.prepared = static_cast<const unsigned char*>(prepared_tree);
    a.out = out; a.lse = lse; a.status = status;
    a.part_o = workspace;
    a.part_ml = p.total_bytes ? reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + p.part_o_bytes) : nullptr;
    a.B = desc->B; a.M = desc->M; a.Hq = desc->Hq; a.Hkv = desc->Hkv; a.D = desc->D; a.G = p.G;
    a.soft_len = desc->soft_len; a.max_prefix_len = desc->max_prefix_len;
    a.scale = desc->softmax_scale;
    a.inv_M = 1.0f / (float)desc->M;
    a.head_stride = desc->kv_head_stride ? desc->kv_head_stride : desc->D;
    a.tok_stride = desc->kv_token_stride ? desc->kv_token_stride : (int64_t)desc->Hkv * desc->D;
    a.row_blocks = p.row_blocks; a.n_chunks = p.n_chunks; a.rb_per_wg = p.rb_per_wg;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const hipError_t e = (desc->dtype == TV_DTYPE_F32) ? launch_attention_f32(a, s) : launch_attention_bf16(a, s);
    return e == hipSuccess ? TV_OK : TV_ERR_LAUNCH;
}

int tree_verify_attention(const tv_attn_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                          const int64_t* kv_offset, const int32_t* prefix_len, const int32_t* parent,
                          const uint8_t* kind, const void* prepared_tree, void* out, float* lse, int32_t* status,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
    return enqueue_attention(desc, q, k_pool, v_pool, kv_offset, prefix_len, parent, kind, prepared_tree, out, lse,
                             status, workspace, workspace_bytes, hip_stream);
}

// ---- the same call for callers that cannot allocate ------------------------------------------------------------
// The partial results of the key ranges go to a fixed array in the library's own device image instead of a
// caller's workspace.  Every GPU holds its own copy at its own address, looked up once per device (with that
// device current) and remembered; host code only ever uses the looked-up address.
static __device__ __align__(256) unsigned char scratch[TV_NOALLOC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_addr[kMaxDevices];

static int scratch_for_current_device(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TV_ERR_LAUNCH;
    void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TV_ERR_LAUNCH;
        g_scratch_addr[dev].store(p, std::memory_order_release);     // (two threads racing here store the same address)
    }
    *out = p;
    return TV_OK;
}

int tree_verify_attention_noalloc(const tv_attn_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                                  const int64_t* kv_offset, const int32_t* prefix_len, const int32_t* parent,
                                  const uint8_t* kind, const void* prepared_tree, void* out, float* lse,
                                  int32_t* status, void* hip_stream) {
    const int rc = check_attn_desc(desc);
    if (rc != TV_OK) return rc;
    AttnPlan p;
    const int prc = plan_attention(*desc, &p);
    if (prc != TV_OK) return prc;
    if (p.total_bytes > (size_t)TV_NOALLOC_SCRATCH_BYTES) return TV_ERR_WORKSPACE;     // larger than the fixed array
    void* ws = nullptr;
    const int src = scratch_for_current_device(&ws);
    if (src != TV_OK) return src;
    return enqueue_attention(desc, q, k_pool, v_pool, kv_offset, prefix_len, parent, kind, prepared_tree, out, lse,
                             status, ws, (size_t)TV_NOALLOC_SCRATCH_BYTES, hip_stream);
}

static int check_accept_desc(const tv_accept_desc* d) {
    if (!d || d->struct_size != sizeof(tv_accept_desc)) return TV_ERR_INVALID_ARG;
    if (d->B < 1 || d->T < 1 || d->T > TV_MAX_ROWS || d->V < 1 || d->C < 0) return TV_ERR_INVALID_ARG;
    if (d->rule < TV_RULE_GREEDY || d->rule > TV_RULE_SAMPLE_MATCH) return TV_ERR_INVALID_ARG;
    if (d->rule != TV_RULE_GREEDY && !(d->temperature > 0.f)) return TV_ERR_INVALID_ARG;
    if (d->logits_row_stride != 0 && d->logits_row_stride < d->V) return TV_ERR_INVALID_ARG;
    if (d->logits_dtype != TV_DTYPE_F32 && d->logits_dtype != TV_DTYPE_BF16) return TV_ERR_INVALID_ARG;
    if (d->reserved != 0) return TV_ERR_INVALID_ARG;
    if ((int64_t)d->B * d->T > 65535) return TV_ERR_INVALID_ARG;       // grid dimension limits
    return TV_OK;
}

int tv_accept_workspace_bytes(const tv_accept_desc* desc, size_t* out_bytes) {
    if (!out_bytes) return TV_ERR_INVALID_ARG;
    const int rc = check_accept_desc(desc);
    if (rc != TV_OK) return rc;
    AcceptPlan p;
    const int prc = plan_accept(*desc, &p);
    if (prc != TV_OK) return prc;
    *out_bytes = p.total_bytes;
    return TV_OK;
}

int tree_accept(const tv_accept_desc* desc, const void* target_logits, const void* draft_logits,
                const int32_t* token, const int32_t* parent, const float* uniforms, const int32_t* con_anchor,
                int32_t* path, int32_t* n_accepted, int32_t* final_token, int32_t* final_kind,
                int32_t* last_node, int32_t* selected_con, int32_t* status, void* workspace,
                size_t workspace_bytes, void* hip_stream) {
    const int rc = check_accept_desc(desc);
    if (rc != TV_OK) return rc;
    if (!target_logits || !token || !parent || !path || !n_accepted || !final_token || !final_kind ||
        !last_node || !status)
        return TV_ERR_INVALID_ARG;
    const bool draft_rule = (desc->rule == TV_RULE_DRAFT_WOR || desc->rule == TV_RULE_DRAFT_WR);
    if (draft_rule && !draft_logits) return TV_ERR_INVALID_ARG;
    if (desc->rule != TV_RULE_GREEDY && !uniforms) return TV_ERR_INVALID_ARG;
    if (desc->C > 0 && !con_anchor) return TV_ERR_INVALID_ARG;
    AcceptPlan p;
    const int prc = plan_accept(*desc, &p);
    if (prc != TV_OK) return prc;
    if (!workspace || workspace_bytes < p.total_bytes || ((uintptr_t)workspace & 255)) return TV_ERR_WORKSPACE;
    AcceptArgs a{};
    a.target = target_logits; a.draft = draft_rule ? draft_logits : nullptr;
    a.logits_bf16 = (desc->logits_dtype == TV_DTYPE_BF16) ? 1 : 0;
    a.token = token; a.parent = parent; a.uniforms = uniforms; a.con_anchor = con_anchor;
    a.path = path; a.n_accepted = n_accepted; a.final_token = final_token; a.final_kind = final_kind;
    a.last_node = last_node; a.selected_con = selected_con; a.status = status;
    unsigned char* w = static_cast<unsigned char*>(workspace);
    a.stats = reinterpret_cast<RowStat*>(w);
    w += p.stats_bytes;
    a.z_tok = reinterpret_cast<float*>(w);
    w += p.ztok_bytes;
    a.chain_z = reinterpret_cast<double*>(w);
    w += p.chain_bytes;
    a.accept_bit = reinterpret_cast<int32_t*>(w);
    a.sampled = a.accept_bit;
    w += p.bits_bytes;
    a.chain_parts = reinterpret_cast<unsigned long long*>(w);
    a.B = desc->B; a.T = desc->T; a.V = desc->V; a.C = con_anchor ? desc->C : 0; a.rule = desc->rule;
    a.temperature = desc->temperature;
    a.row_stride = desc->logits_row_stride ? desc->logits_row_stride : desc->V;
    a.splits = p.splits; a.split_len = p.split_len; a.n_mat = p.n_mat;
    a.chain_slices = p.chain_slices;
    const int wl = g_wait_limit.load();
    a.wait_limit = wl > 0 ? (unsigned)wl : (1u << 20);
    const hipError_t e = launch_accept(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TV_OK : TV_ERR_LAUNCH;
}

int tree_commit(const tv_commit_desc* d, void* k_pool, void* v_pool, const int64_t* kv_offset,
                const int32_t* prefix_len, const int32_t* path, const int32_t* n_accepted, const int32_t* node_row,
                const void* hidden, const int32_t* con_row, const int32_t* selected_con, void* f_out,
                int32_t* new_prefix_len, int32_t* status, void* hip_stream) {
    if (!d || d->struct_size != sizeof(tv_commit_desc)) return TV_ERR_INVALID_ARG;
    if (d->dtype != TV_DTYPE_F32 && d->dtype != TV_DTYPE_BF16) return TV_ERR_INVALID_ARG;
    const int elem = (d->dtype == TV_DTYPE_F32) ? 4 : 2;
    if (d->B < 1 || d->B > 65535 || d->T < 1 || d->T > TV_MAX_ROWS || d->M < d->T || d->M > TV_MAX_ROWS) return TV_ERR_INVALID_ARG;
    if (d->Hkv < 1 || d->D < 1 || (d->D * elem) % 16 != 0 || d->n_layers < 1 || d->n_layers > 65535) return TV_ERR_INVALID_ARG;
    if (d->C < 0 || d->d_model < 0 || (d->d_model * elem) % 16 != 0) return TV_ERR_INVALID_ARG;
    if (d->kv_token_stride < 0 || d->kv_head_stride < 0 || d->kv_layer_stride < 0) return TV_ERR_INVALID_ARG;
    const int64_t hs = d->kv_head_stride ? d->kv_head_stride : d->D;
    const int64_t ts = d->kv_token_stride ? d->kv_token_stride : (int64_t)d->Hkv * d->D;
    if (hs < d->D || ts < d->D || (hs * elem) % 16 != 0 || (ts * elem) % 16 != 0) return TV_ERR_INVALID_ARG;
    if (d->n_layers > 1 && (d->kv_layer_stride <= 0 || (d->kv_layer_stride * elem) % 16 != 0)) return TV_ERR_INVALID_ARG;
    if (!k_pool || !v_pool || !kv_offset || !prefix_len || !path || !n_accepted || !new_prefix_len || !status)
        return TV_ERR_INVALID_ARG;
    if (((uintptr_t)k_pool | (uintptr_t)v_pool) & 15) return TV_ERR_INVALID_ARG;
    const bool gather = hidden != nullptr;
    if (gather && (!con_row || !selected_con || !f_out || d->d_model < 1 || d->C < 1)) return TV_ERR_INVALID_ARG;
    if (gather && (((uintptr_t)hidden | (uintptr_t)f_out) & 15)) return TV_ERR_INVALID_ARG;
    CommitArgs a{};
    a.k = k_pool; a.v = v_pool; a.kv_offset = kv_offset; a.prefix_len = prefix_len; a.path = path;
    a.n_accepted = n_accepted; a.node_row = node_row;
    a.hidden = hidden; a.con_row = gather ? con_row : nullptr; a.selected_con = gather ? selected_con : nullptr;
    a.f_out = gather ? f_out : nullptr;
    a.new_prefix_len = new_prefix_len; a.status = status;
    a.B = d->B; a.T = d->T; a.M = d->M; a.Hkv = d->Hkv; a.D = d->D; a.n_layers = d->n_layers; a.C = d->C;
    a.d_model = d->d_model; a.elem = elem;
    a.layer_stride = d->n_layers > 1 ? d->kv_layer_stride : 0; a.tok_stride = ts; a.head_stride = hs;
    const hipError_t e = launch_commit(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TV_OK : TV_ERR_LAUNCH;
}

static int check_embed_desc(const tv_embed_desc* d) {
    if (!d || d->struct_size != sizeof(tv_embed_desc)) return TV_ERR_INVALID_ARG;
    if (d->dtype != TV_DTYPE_F32 && d->dtype != TV_DTYPE_BF16) return TV_ERR_INVALID_ARG;
    if (d->B < 1 || d->B > 65535 || d->d_in < 8 || d->d_in % 8 != 0 || d->d_out < 8 || d->d_out % 8 != 0)
        return TV_ERR_INVALID_ARG;
    if (d->n_expert < 1 || d->n_expert > 64 || d->k_expert < 1 || d->k_expert > d->n_expert || d->reserved != 0)
        return TV_ERR_INVALID_ARG;
    return TV_OK;
}

int tv_embed_workspace_bytes(const tv_embed_desc* desc, size_t* out_bytes) {
    if (!out_bytes) return TV_ERR_INVALID_ARG;
    const int rc = check_embed_desc(desc);
    if (rc != TV_OK) return rc;
    *out_bytes = up256((size_t)desc->B * desc->n_expert * sizeof(float));
    return TV_OK;
}

int contemplate_embed(const tv_embed_desc* d, const void* h, const void* router_w, const void* expert_emb, void* out,
                      float* gates, int32_t* chosen, void* workspace, size_t workspace_bytes, void* hip_stream) {
    const int rc = check_embed_desc(d);
    if (rc != TV_OK) return rc;
    if (!workspace || workspace_bytes < up256((size_t)d->B * d->n_expert * sizeof(float)) || ((uintptr_t)workspace & 15))
        return TV_ERR_WORKSPACE;
    if (!h || !router_w || !expert_emb || !out) return TV_ERR_INVALID_ARG;
    if (((uintptr_t)h | (uintptr_t)router_w | (uintptr_t)expert_emb | (uintptr_t)out) & 15) return TV_ERR_INVALID_ARG;
    EmbedArgs a{};
    a.h = h; a.router_w = router_w; a.expert_emb = expert_emb; a.out = out; a.gates = gates; a.chosen = chosen;
    a.logits = static_cast<float*>(workspace);
    a.B = d->B; a.d_in = d->d_in; a.d_out = d->d_out; a.n_expert = d->n_expert; a.k_expert = d->k_expert;
    a.bf16 = (d->dtype == TV_DTYPE_BF16);
    const hipError_t e = launch_embed(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TV_OK : TV_ERR_LAUNCH;
}

}  // extern "C"
