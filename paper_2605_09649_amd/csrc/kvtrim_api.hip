// C ABI of libkvtrim: argument checks, workspace, and dispatch to the kernel launchers.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "kvtrim_internal.h"

namespace kvtrim {

kvtrim_status hip_fail(kvtrim_ctx* ctx, hipError_t e, const char* what) {
    if (ctx) snprintf(ctx->last_error, sizeof(ctx->last_error), "%s: %s", what, hipGetErrorString(e));
    return KVTRIM_EHIP;
}

static kvtrim_status invalid(kvtrim_ctx* ctx, const char* why) {
    if (ctx) snprintf(ctx->last_error, sizeof(ctx->last_error), "invalid argument: %s", why);
    return KVTRIM_EINVAL;
}

static bool config_ok(const kvtrim_config* c) {
    if (!c) return false;
    if (c->n_seq < 1 || c->n_layers < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1) return false;
    if (c->n_q_heads % c->n_kv_heads) return false;
    const int g = c->n_q_heads / c->n_kv_heads;
    if (g < 1 || g > 8) return false;
    if (c->head_dim != 64 && c->head_dim != 128) return false;
    if (c->max_entries < 1 || c->max_entries > ((int64_t)1 << 31) - 4096) return false;
    const int64_t nseg = (int64_t)c->n_seq * c->n_layers * c->n_kv_heads;
    if (nseg > (1 << 24) || c->n_seq > 65536) return false;
    return true;
}

struct Layout {
    size_t off[41];
    int32_t fl_cap;
    size_t total;
    int64_t max_sel_chunks, max_cmp_chunks, max_att_chunks, gat_slots;
};

static size_t bump(size_t& cur, size_t bytes) {
    size_t at = (cur + 255) & ~(size_t)255;
    cur = at + bytes;
    return at;
}

// select_only: the arrays of the compaction and the attention get no room (a workspace for stage 2 alone).
static Layout layout_of(const kvtrim_config* c, bool select_only) {
    Layout l;
    const int64_t nseg = (int64_t)c->n_seq * c->n_layers * c->n_kv_heads;
    const int G = c->n_q_heads / c->n_kv_heads;
    l.max_sel_chunks = c->max_entries / SEL_CHUNK + nseg;
    l.max_cmp_chunks = select_only ? 0 : c->max_entries / CMP_CHUNK + nseg;
    // the attention chunk grows with the capacity (att_chunk_for) so that at most 16384 full
    // chunks plus one ragged tail per segment ever exist
    // (the fused stage 3+4 kernel also writes one partial result per 128-entry compaction chunk;
    // it is used for caches of up to 524288 such chunks = 67 M entries, larger ones take the two-call path;
    // the buffer is [chunk][G][D + 2] fp32, 2 KB per chunk at G = 4, D = 128)
    const int64_t full = c->max_entries / CMP_CHUNK < 524288 ? c->max_entries / CMP_CHUNK : 524288;
    const int64_t att = select_only ? 0 : full + nseg + 1;
    l.max_att_chunks = att;
    const size_t seg_tables = select_only ? 0 : 1;                             // per-segment arrays the selection does not use
    size_t cur = 0;
    l.off[0] = bump(cur, (nseg + 1) * sizeof(int32_t));                        // sel_chunk_prefix
    l.off[1] = bump(cur, l.max_sel_chunks * sizeof(ChunkDesc));                // sel_desc
    l.off[2] = bump(cur, (size_t)3 * HIST_REPLICAS * c->n_seq * RADIX_BINS * sizeof(uint32_t)); // hist
    l.off[3] = bump(cur, (size_t)4 * c->n_seq * sizeof(SelState));             // sel: final state + the state after the plan and after each of the first two passes
    l.off[4] = bump(cur, DONE_WORDS * sizeof(uint32_t));                       // done
    l.off[5] = bump(cur, l.max_sel_chunks * sizeof(int32_t));                  // chunk_eq
    l.off[6] = bump(cur, l.max_sel_chunks * sizeof(int64_t));                  // chunk_tie_base
    l.off[7] = bump(cur, seg_tables * (nseg + 1) * sizeof(int32_t));           // cmp_chunk_prefix
    l.off[8] = bump(cur, l.max_cmp_chunks * sizeof(ChunkDesc));                // cmp_desc
    l.off[9] = bump(cur, l.max_cmp_chunks * sizeof(int64_t));                  // cmp_chunk_dst
    l.off[10] = bump(cur, seg_tables * (nseg + 1) * sizeof(int32_t));          // att_chunk_prefix
    l.off[11] = bump(cur, l.max_att_chunks * sizeof(ChunkDesc));               // att_desc
    l.off[12] = bump(cur, (size_t)l.max_att_chunks * G * (c->head_dim + 2) * sizeof(float)); // att_partial
    l.off[13] = bump(cur, 256);                                                // err (word 0), fast_stat (bytes 64..79)
    l.off[14] = bump(cur, (nseg + 1) * sizeof(int64_t));                       // sel_entry_prefix
    l.off[15] = bump(cur, HIST_BLOCKS_MAX * sizeof(int4));                     // sel_blk
    l.off[16] = bump(cur, seg_tables * (size_t)nseg * sizeof(int32_t));        // tie_cnt
    l.off[17] = bump(cur, seg_tables * (size_t)nseg * sizeof(int32_t));        // tie_mode
    l.off[18] = bump(cur, seg_tables * (size_t)nseg * sizeof(int32_t));        // tie_thr
    l.off[19] = bump(cur, seg_tables * (size_t)nseg * sizeof(int64_t));        // pg_seg_start
    l.off[20] = bump(cur, seg_tables * (size_t)nseg * sizeof(int32_t));        // pg_seg_len
    l.off[21] = bump(cur, (size_t)c->n_seq * sizeof(uint32_t));                // seq_done
    l.off[22] = bump(cur, seg_tables * (size_t)nseg * sizeof(int32_t));        // chunk_old_len
    // decode-step selection: a candidate list per sequence, shorter when there are many sequences (1 M entries in all)
    int64_t fl = ((int64_t)1 << 20) / c->n_seq / 64 * 64;
    fl = fl > FL_CAP_MAX ? FL_CAP_MAX : (fl < FL_CAP_MIN ? FL_CAP_MIN : fl);
    l.fl_cap = select_only ? 0 : (int32_t)fl;
    l.off[24] = bump(cur, seg_tables * (size_t)c->n_seq * sizeof(uint32_t));   // fast_hi
    l.off[25] = bump(cur, seg_tables * (size_t)c->n_seq * 16 * sizeof(uint32_t));   // fast_min: 16 group words per sequence
    l.off[26] = bump(cur, seg_tables * (size_t)c->n_seq * 17 * sizeof(uint32_t));   // fast_done: top-level + 16 group counters
    l.off[27] = bump(cur, seg_tables * (size_t)c->n_seq * 16 * sizeof(uint32_t));   // fl_count: one per sub-list
    l.off[28] = bump(cur, seg_tables * (size_t)c->n_seq * sizeof(FastSel));    // fast_sel
    l.off[29] = bump(cur, (size_t)c->n_seq * l.fl_cap * sizeof(uint32_t));     // fl_key
    l.off[30] = bump(cur, (size_t)c->n_seq * l.fl_cap * sizeof(int32_t));      // fl_seg
    l.off[31] = bump(cur, (size_t)c->n_seq * l.fl_cap * sizeof(int32_t));      // fl_pos
    l.off[32] = bump(cur, (size_t)c->n_seq * l.fl_cap * sizeof(int32_t));      // fl_idx
    l.off[33] = bump(cur, seg_tables * (size_t)nseg * sizeof(int32_t));        // step_len
    l.off[34] = bump(cur, l.max_att_chunks * 4 * sizeof(int32_t));             // att_pages
    l.off[35] = bump(cur, seg_tables * (size_t)nseg * sizeof(StepSegRec));     // step_rec
    l.off[36] = bump(cur, seg_tables * (size_t)c->n_seq * STEP_MAX_EVICT * sizeof(int32_t));   // step_evl
    l.off[37] = bump(cur, (size_t)l.max_cmp_chunks * sizeof(uint32_t));        // step_chunk_ev
    // a destination under a quarter of the source: at most max_entries / 4 rows in chunks of CMP_CHUNK, one ragged chunk per segment
    l.gat_slots = select_only ? 0 : c->max_entries / 4 + ((int64_t)nseg + 1) * CMP_CHUNK;
    l.off[38] = bump(cur, (size_t)l.gat_slots * sizeof(int32_t));              // gat_src
    l.off[39] = bump(cur, seg_tables * (size_t)(nseg + 1) * sizeof(int64_t));  // att_row_prefix
    l.off[40] = bump(cur, (size_t)c->n_layers * sizeof(uint32_t));             // gate_done
    l.total = (cur + 255) & ~(size_t)255;
    return l;
}

static void bind(const Layout& l, char* b, Workspace& w) {
    w.sel_chunk_prefix = (int32_t*)(b + l.off[0]);
    w.sel_desc = (ChunkDesc*)(b + l.off[1]);
    w.hist = (uint32_t*)(b + l.off[2]);
    w.sel = (SelState*)(b + l.off[3]);
    w.done = (uint32_t*)(b + l.off[4]);
    w.chunk_eq = (int32_t*)(b + l.off[5]);
    w.chunk_tie_base = (int64_t*)(b + l.off[6]);
    w.cmp_chunk_prefix = (int32_t*)(b + l.off[7]);
    w.cmp_desc = (ChunkDesc*)(b + l.off[8]);
    w.cmp_chunk_dst = (int64_t*)(b + l.off[9]);
    w.att_chunk_prefix = (int32_t*)(b + l.off[10]);
    w.att_desc = (ChunkDesc*)(b + l.off[11]);
    w.att_partial = (float*)(b + l.off[12]);
    w.pg_block_table = nullptr;
    w.err = (int32_t*)(b + l.off[13]);
    w.fast_stat = (unsigned long long*)(b + l.off[13] + 64);
    w.sel_entry_prefix = (int64_t*)(b + l.off[14]);
    w.sel_blk = (int4*)(b + l.off[15]);
    w.tie_cnt = (int32_t*)(b + l.off[16]);
    w.tie_mode = (int32_t*)(b + l.off[17]);
    w.tie_thr = (int32_t*)(b + l.off[18]);
    w.pg_seg_start = (int64_t*)(b + l.off[19]);
    w.pg_seg_len = (int32_t*)(b + l.off[20]);
    w.seq_done = (uint32_t*)(b + l.off[21]);
    w.chunk_old_len = (int32_t*)(b + l.off[22]);
    w.fast_hi = (uint32_t*)(b + l.off[24]);
    w.fast_min = (uint32_t*)(b + l.off[25]);
    w.fast_done = (uint32_t*)(b + l.off[26]);
    w.fl_count = (uint32_t*)(b + l.off[27]);
    w.fast_sel = (FastSel*)(b + l.off[28]);
    w.fl_key = (uint32_t*)(b + l.off[29]);
    w.fl_seg = (int32_t*)(b + l.off[30]);
    w.fl_pos = (int32_t*)(b + l.off[31]);
    w.fl_idx = (int32_t*)(b + l.off[32]);
    w.step_len = (int32_t*)(b + l.off[33]);
    w.att_pages = (int32_t*)(b + l.off[34]);
    w.step_rec = (StepSegRec*)(b + l.off[35]);
    w.step_evl = (int32_t*)(b + l.off[36]);
    w.step_chunk_ev = (uint32_t*)(b + l.off[37]);
    w.gat_src = (int32_t*)(b + l.off[38]);
    w.att_row_prefix = (int64_t*)(b + l.off[39]);
    w.gate_done = (uint32_t*)(b + l.off[40]);
    w.gat_slots = l.gat_slots;
    w.fl_cap = l.fl_cap;
    w.max_sel_chunks = l.max_sel_chunks;
    w.max_cmp_chunks = l.max_cmp_chunks;
    w.max_att_chunks = l.max_att_chunks;
}

bool config_valid(const kvtrim_config* c) { return config_ok(c); }

void shape_of(const kvtrim_config* cfg, Shape& sh) {
    sh.n_seq = cfg->n_seq;
    sh.n_layers = cfg->n_layers;
    sh.n_kv_heads = cfg->n_kv_heads;
    sh.n_q_heads = cfg->n_q_heads;
    sh.head_dim = cfg->head_dim;
    sh.segs_per_seq = cfg->n_layers * cfg->n_kv_heads;
    sh.nseg = cfg->n_seq * sh.segs_per_seq;
    sh.group = cfg->n_q_heads / cfg->n_kv_heads;
}

size_t select_workspace(const kvtrim_config* cfg, char* base, Workspace* ws) {
    const Layout l = layout_of(cfg, true);
    if (ws) bind(l, base, *ws);
    return l.total;
}

static CacheView view_of(const kvtrim_cache* c) {
    CacheView v;
    v.k = (const uint16_t*)c->k;
    v.v = (const uint16_t*)c->v;
    v.log_beta = c->log_beta;
    v.pos = c->pos;
    v.seg_start = c->seg_start;
    v.seg_len = c->seg_len;
    v.cap = c->cap_entries;
    v.log_tail = c->log_tail;
    return v;
}

static CacheViewMut view_mut_of(const kvtrim_cache* c) {
    CacheViewMut v;
    v.k = (uint16_t*)c->k;
    v.v = (uint16_t*)c->v;
    v.log_beta = c->log_beta;
    v.pos = c->pos;
    v.seg_start = c->seg_start;
    v.seg_len = c->seg_len;
    v.cap = c->cap_entries;
    v.log_tail = c->log_tail;
    return v;
}

static const char* cache_problem(const kvtrim_ctx* ctx, const kvtrim_cache* c, bool need_rows) {
    if (!c) return "cache is NULL";
    if (!c->log_beta || !c->pos || !c->seg_start || !c->seg_len) return "cache has a NULL metadata pointer";
    if (need_rows && (!c->k || !c->v)) return "cache has a NULL k/v pointer";
    if (need_rows && ((((uintptr_t)c->k) | ((uintptr_t)c->v)) & 15)) return "k/v not 16-byte aligned";
    if (c->cap_entries < 1 || c->cap_entries > ctx->cfg.max_entries) return "cap_entries outside [1, max_entries]";
    return nullptr;
}

}  // namespace kvtrim

using namespace kvtrim;

extern "C" {

size_t kvtrim_workspace_bytes(const kvtrim_config* cfg) {
    if (!config_ok(cfg)) return 0;
    return layout_of(cfg, false).total;
}

// Why the calling thread's last kvtrim_create failed (there is no context to hold the text).
static thread_local char g_create_error[256] = "no context";

kvtrim_status kvtrim_create(kvtrim_ctx** out, const kvtrim_config* cfg) {
    if (!out) return KVTRIM_EINVAL;
    *out = nullptr;
    if (!config_ok(cfg)) {
        snprintf(g_create_error, sizeof g_create_error, "kvtrim_create: configuration out of range");
        return KVTRIM_EINVAL;
    }
    kvtrim_ctx* ctx = new (std::nothrow) kvtrim_ctx;
    if (!ctx) {
        snprintf(g_create_error, sizeof g_create_error, "kvtrim_create: no host memory for the context");
        return KVTRIM_ENOMEM;
    }
    memset(ctx, 0, sizeof(*ctx));
    ctx->cfg = *cfg;
    shape_of(cfg, ctx->shape);
    ctx->att_chunk_min = 512;
    if (const char* e = getenv("KVTRIM_ATT_CHUNK")) {            // tuning knob: rows per attention chunk
        const int v = atoi(e);
        if (v >= 256 && v <= 65536 && v % 64 == 0) ctx->att_chunk_min = v;
    }
    ctx->att_blocks = 768;                                        // three blocks of k_att_partial per compute unit
    if (const char* e = getenv("KVTRIM_ATT_BLOCKS")) {           // tuning knob
        const int v = atoi(e);
        if (v >= 1 && v <= 65536) ctx->att_blocks = v;
    }
    const Layout l = layout_of(cfg, false);
    ctx->ws_bytes = l.total;
    hipError_t e = hipGetDevice(&ctx->device);
    if (e != hipSuccess) {
        snprintf(g_create_error, sizeof g_create_error, "kvtrim_create: hipGetDevice: %s", hipGetErrorString(e));
        (void)hipGetLastError();
        delete ctx;
        return KVTRIM_EHIP;
    }
    e = hipMalloc(&ctx->ws_base, l.total);
    if (e != hipSuccess) {                                        // (an earlier asynchronous failure is reported here too)
        snprintf(g_create_error, sizeof g_create_error, "kvtrim_create: hipMalloc of the %zu-byte workspace: %s", l.total,
                 hipGetErrorString(e));
        (void)hipGetLastError();
        delete ctx;
        return e == hipErrorOutOfMemory ? KVTRIM_ENOMEM : KVTRIM_EHIP;
    }
    if ((e = hipHostMalloc((void**)&ctx->err_host, sizeof(int32_t), hipHostMallocDefault)) != hipSuccess ||
        (e = hipMemset(ctx->ws_base, 0, l.total)) != hipSuccess ||
        (e = hipMemset((char*)ctx->ws_base + l.off[25], 0xFF, (size_t)cfg->n_seq * 16 * sizeof(uint32_t))) != hipSuccess ||   // fast_min: "no key seen"
        (e = hipDeviceSynchronize()) != hipSuccess) {
        snprintf(g_create_error, sizeof g_create_error, "kvtrim_create: setting up the workspace: %s", hipGetErrorString(e));
        (void)hipGetLastError();
        if (ctx->err_host) (void)hipHostFree(ctx->err_host);
        (void)hipFree(ctx->ws_base);
        delete ctx;
        return KVTRIM_EHIP;
    }
    bind(l, (char*)ctx->ws_base, ctx->ws);
    *out = ctx;
    return KVTRIM_OK;
}

static void free_profile(kvtrim_ctx* ctx) {
    if (ctx->prof_ev) {
        for (int i = 0; i < 2 * KVTRIM_PROFILE_MAX_LAUNCHES; ++i)
            if (ctx->prof_ev[i]) (void)hipEventDestroy(ctx->prof_ev[i]);
        delete[] ctx->prof_ev;
        ctx->prof_ev = nullptr;
    }
    delete[] ctx->prof_kernel;
    ctx->prof_kernel = nullptr;
    ctx->prof_mask = 0;
    ctx->prof_used = 0;
}

static const char* const kernel_names[KVTRIM_N_KERNELS] = {
    "k_score", "k_sel_plan", "k_sel_hist<0>", "k_sel_hist<1>", "k_sel_hist<2>", "k_sel_count", "k_sel_mask",
    "k_cmp_scan", "k_cmp_copy", "k_att_plan", "k_att_partial", "k_att_combine", "k_append", "k_cmp_attn", "k_occupancy",
    "k_pg_init", "k_pg_append", "k_pg_score", "k_pg_plan", "k_pg_count", "k_pg_evict", "k_pg_tidy", "k_pg_att_plan", "k_gate_hidden", "k_gate_readout",
    "k_gate_fold", "k_gate_prefill", "k_gate_retile", "k_pg_defrag", "k_gate_dot", "reserved30", "k_cmp_unstage",
    "k_fast_scan", "k_fast_mask", "reserved34", "reserved35", "reserved36", "reserved37", "reserved38", "reserved39"};

const char* kvtrim_kernel_name(int32_t id) { return id >= 0 && id < KVTRIM_N_KERNELS ? kernel_names[id] : nullptr; }

kvtrim_status kvtrim_profile_begin(kvtrim_ctx* ctx, uint64_t kernel_mask) {
    if (!ctx) return KVTRIM_EINVAL;
    if (!ctx->prof_ev) {
        ctx->prof_ev = new (std::nothrow) hipEvent_t[2 * KVTRIM_PROFILE_MAX_LAUNCHES]();
        ctx->prof_kernel = new (std::nothrow) int8_t[KVTRIM_PROFILE_MAX_LAUNCHES]();
        if (!ctx->prof_ev || !ctx->prof_kernel) {
            free_profile(ctx);
            return KVTRIM_ENOMEM;
        }
        for (int i = 0; i < 2 * KVTRIM_PROFILE_MAX_LAUNCHES; ++i) {
            hipError_t e = hipEventCreate(&ctx->prof_ev[i]);
            if (e != hipSuccess) {
                free_profile(ctx);
                return hip_fail(ctx, e, "hipEventCreate");
            }
        }
    }
    ctx->prof_used = 0;
    ctx->prof_mask = kernel_mask;
    return KVTRIM_OK;
}

kvtrim_status kvtrim_profile_end(kvtrim_ctx* ctx, void* hip_stream, double* ms_sum, int64_t* launches) {
    if (!ctx || !ms_sum || !launches) return KVTRIM_EINVAL;
    ctx->prof_mask = 0;
    for (int i = 0; i < KVTRIM_N_KERNELS; ++i) {
        ms_sum[i] = 0.0;
        launches[i] = 0;
    }
    KVTRIM_HIP(ctx, hipStreamSynchronize((hipStream_t)hip_stream));
    for (int s = 0; s < ctx->prof_used; ++s) {
        float ms = 0.f;
        KVTRIM_HIP(ctx, hipEventElapsedTime(&ms, ctx->prof_ev[2 * s], ctx->prof_ev[2 * s + 1]));
        ms_sum[ctx->prof_kernel[s]] += ms;
        launches[ctx->prof_kernel[s]] += 1;
    }
    ctx->prof_used = 0;
    return KVTRIM_OK;
}

kvtrim_status kvtrim_destroy(kvtrim_ctx* ctx) {
    if (!ctx) return KVTRIM_EINVAL;
    (void)hipDeviceSynchronize();
    free_profile(ctx);
    if (ctx->err_host) (void)hipHostFree(ctx->err_host);
    if (ctx->ws_base) (void)hipFree(ctx->ws_base);
    delete ctx;
    return KVTRIM_OK;
}

const char* kvtrim_last_error(const kvtrim_ctx* ctx) { return ctx ? ctx->last_error : g_create_error; }

kvtrim_status kvtrim_poll_error(kvtrim_ctx* ctx, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    KVTRIM_HIP(ctx, hipMemcpyAsync(ctx->err_host, ctx->ws.err, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    KVTRIM_HIP(ctx, hipStreamSynchronize(st));
    const int32_t e = *ctx->err_host;
    if (e) {
        *ctx->err_host = 0;
        KVTRIM_HIP(ctx, hipMemcpyAsync(ctx->ws.err, ctx->err_host, sizeof(int32_t), hipMemcpyHostToDevice, st));
        KVTRIM_HIP(ctx, hipStreamSynchronize(st));
    }
    if (e & ERR_LAYOUT) return KVTRIM_ELAYOUT;
    if (e & ERR_CAP) return KVTRIM_ECAP;
    if (e & ERR_MISMATCH) return KVTRIM_EMISMATCH;
    return KVTRIM_OK;
}

kvtrim_status kvtrim_score(kvtrim_ctx* ctx, const kvtrim_cache* c, const int32_t* now, float* score_out,
                           void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, c, false)) return invalid(ctx, p);
    if (!now || !score_out) return invalid(ctx, "now / score_out is NULL");
    return launch_score(ctx, view_of(c), now, score_out, (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_select_global(kvtrim_ctx* ctx, const kvtrim_cache* c, const float* score,
                                   const int64_t* budget, uint8_t* keep_out, int32_t* kept_out,
                                   uint32_t* thr_key_out, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, c, false)) return invalid(ctx, p);
    if (!score || !budget || !keep_out || !kept_out) return invalid(ctx, "score / budget / keep_out / kept_out is NULL");
    return launch_select(ctx, view_of(c), score, budget, keep_out, kept_out, thr_key_out, (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_select_path_counts(kvtrim_ctx* ctx, int64_t* from_list_host, int64_t* fallback_host, void* hip_stream) {
    if (!ctx || !from_list_host || !fallback_host) return KVTRIM_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    unsigned long long v[2] = {0, 0};
    KVTRIM_HIP(ctx, hipStreamSynchronize(st));
    KVTRIM_HIP(ctx, hipMemcpy(v, ctx->ws.fast_stat, sizeof(v), hipMemcpyDeviceToHost));
    *from_list_host = (int64_t)v[0];
    *fallback_host = (int64_t)v[1];
    return KVTRIM_OK;
}

kvtrim_status kvtrim_score_select(kvtrim_ctx* ctx, const kvtrim_cache* c, const int32_t* now, const int64_t* budget,
                                  float* score_out, uint8_t* keep_out, int32_t* kept_out, uint32_t* thr_key_out,
                                  int64_t evict_hint, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, c, false)) return invalid(ctx, p);
    if (!now || !budget || !score_out || !keep_out || !kept_out)
        return invalid(ctx, "now / budget / score_out / keep_out / kept_out is NULL");
    return launch_score_select(ctx, view_of(c), now, budget, score_out, keep_out, kept_out, thr_key_out,
                               evict_hint, (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_compact(kvtrim_ctx* ctx, const kvtrim_cache* src, const uint8_t* keep, const int32_t* kept,
                             kvtrim_cache* dst, int32_t reserve, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, src, true)) return invalid(ctx, p);
    if (const char* p = cache_problem(ctx, dst, true)) return invalid(ctx, p);
    if (!keep || !kept) return invalid(ctx, "keep / kept is NULL");
    if (reserve < 0) return invalid(ctx, "reserve < 0");
    if (src->k == dst->k || src->v == dst->v || src->log_beta == dst->log_beta || src->pos == dst->pos ||
        src->seg_start == dst->seg_start || src->seg_len == dst->seg_len)
        return invalid(ctx, "src and dst share a buffer");
    if ((src->log_tail == nullptr) != (dst->log_tail == nullptr) || (src->log_tail && src->log_tail == dst->log_tail))
        return invalid(ctx, "log_tail must be set in both caches or in neither, and not shared");
    return launch_compact(ctx, view_of(src), keep, kept, view_mut_of(dst), reserve, (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_decode_attn(kvtrim_ctx* ctx, const kvtrim_cache* c, const void* q, int32_t layer_begin,
                                 int32_t layer_end, float softmax_scale, float* out, float* lse,
                                 void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, c, true)) return invalid(ctx, p);
    if (!q || !out) return invalid(ctx, "q / out is NULL");
    if (((uintptr_t)q) & 15) return invalid(ctx, "q not 16-byte aligned");
    if (layer_begin < 0 || layer_end > ctx->cfg.n_layers || layer_begin >= layer_end)
        return invalid(ctx, "empty or out-of-range layer range");
    if (!(softmax_scale == softmax_scale)) return invalid(ctx, "softmax_scale is NaN");
    return launch_attn(ctx, view_of(c), (const uint16_t*)q, nullptr, layer_begin, layer_end, softmax_scale, out, lse,
                       (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_decode_attn_soft(kvtrim_ctx* ctx, const kvtrim_cache* c, const void* q, const int32_t* now,
                                      int32_t layer_begin, int32_t layer_end, float softmax_scale, float* out,
                                      float* lse, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, c, true)) return invalid(ctx, p);
    if (!q || !out || !now) return invalid(ctx, "q / out / now is NULL");
    if (((uintptr_t)q) & 15) return invalid(ctx, "q not 16-byte aligned");
    if (layer_begin < 0 || layer_end > ctx->cfg.n_layers || layer_begin >= layer_end)
        return invalid(ctx, "empty or out-of-range layer range");
    if (!(softmax_scale == softmax_scale)) return invalid(ctx, "softmax_scale is NaN");
    return launch_attn(ctx, view_of(c), (const uint16_t*)q, now, layer_begin, layer_end, softmax_scale, out, lse,
                       (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_occupancy(kvtrim_ctx* ctx, const kvtrim_cache* c, const int32_t* now, double* occ_out,
                               void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, c, false)) return invalid(ctx, p);
    if (!now || !occ_out) return invalid(ctx, "now / occ_out is NULL");
    return launch_occupancy(ctx, view_of(c), now, occ_out, (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_compact_attn(kvtrim_ctx* ctx, const kvtrim_cache* src, const uint8_t* keep, const int32_t* kept,
                                  kvtrim_cache* dst, int32_t reserve, const void* q, int32_t layer_begin,
                                  int32_t layer_end, float softmax_scale, float* out, float* lse, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, src, true)) return invalid(ctx, p);
    if (const char* p = cache_problem(ctx, dst, true)) return invalid(ctx, p);
    if (!keep || !kept) return invalid(ctx, "keep / kept is NULL");
    if (reserve < 0) return invalid(ctx, "reserve < 0");
    if (src->k == dst->k || src->v == dst->v || src->log_beta == dst->log_beta || src->pos == dst->pos ||
        src->seg_start == dst->seg_start || src->seg_len == dst->seg_len)
        return invalid(ctx, "src and dst share a buffer");
    if ((src->log_tail == nullptr) != (dst->log_tail == nullptr) || (src->log_tail && src->log_tail == dst->log_tail))
        return invalid(ctx, "log_tail must be set in both caches or in neither, and not shared");
    if (!q || !out) return invalid(ctx, "q / out is NULL");
    if (((uintptr_t)q) & 15) return invalid(ctx, "q not 16-byte aligned");
    if (layer_begin < 0 || layer_end > ctx->cfg.n_layers || layer_begin >= layer_end)
        return invalid(ctx, "empty or out-of-range layer range");
    if (!(softmax_scale == softmax_scale)) return invalid(ctx, "softmax_scale is NaN");
    return launch_compact_attn(ctx, view_of(src), keep, kept, view_mut_of(dst), reserve, (const uint16_t*)q,
                               layer_begin, layer_end, softmax_scale, out, lse, (hipStream_t)hip_stream);
}

// argument checks shared by the two in-place calls; returns NULL when cache, spare, keep and kept are usable
static const char* inplace_problem(const kvtrim_ctx* ctx, const kvtrim_cache* c, const uint8_t* keep, const int32_t* kept,
                                   const kvtrim_cache* spare) {
    if (const char* p = cache_problem(ctx, c, true)) return p;
    if (!spare || !spare->k || !spare->v || !spare->log_beta || !spare->pos) return "spare or one of its k / v / log_beta / pos arrays is NULL";
    if ((((uintptr_t)spare->k) | ((uintptr_t)spare->v)) & 15) return "spare k/v not 16-byte aligned";
    if (spare->cap_entries < c->cap_entries) return "spare holds fewer entries than the cache";
    if (c->k == spare->k || c->v == spare->v || c->log_beta == spare->log_beta || c->pos == spare->pos)
        return "the cache and spare share a buffer";
    if (c->log_tail && (!spare->log_tail || spare->log_tail == c->log_tail))
        return "the cache carries log_tail: spare needs a log_tail array of its own";
    if (!keep || !kept) return "keep / kept is NULL";
    return nullptr;
}

kvtrim_status kvtrim_min_room(kvtrim_ctx* ctx, const kvtrim_cache* c, int32_t* min_room_out, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, c, false)) return invalid(ctx, p);
    if (!min_room_out) return invalid(ctx, "min_room_out is NULL");
    return launch_min_room(ctx, view_of(c), min_room_out, (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_compact_inplace(kvtrim_ctx* ctx, kvtrim_cache* c, const uint8_t* keep, const int32_t* kept,
                                     kvtrim_cache* spare, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = inplace_problem(ctx, c, keep, kept, spare)) return invalid(ctx, p);
    return launch_compact_inplace(ctx, view_mut_of(c), keep, kept, view_mut_of(spare), (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_compact_attn_inplace(kvtrim_ctx* ctx, kvtrim_cache* c, const uint8_t* keep, const int32_t* kept,
                                          kvtrim_cache* spare, const void* q, int32_t layer_begin, int32_t layer_end,
                                          float softmax_scale, float* out, float* lse, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = inplace_problem(ctx, c, keep, kept, spare)) return invalid(ctx, p);
    if (!q || !out) return invalid(ctx, "q / out is NULL");
    if (((uintptr_t)q) & 15) return invalid(ctx, "q not 16-byte aligned");
    if (layer_begin < 0 || layer_end > ctx->cfg.n_layers || layer_begin >= layer_end)
        return invalid(ctx, "empty or out-of-range layer range");
    if (!(softmax_scale == softmax_scale)) return invalid(ctx, "softmax_scale is NaN");
    if (c->cap_entries / CMP_CHUNK + ctx->shape.nseg > ctx->ws.max_att_chunks)
        return invalid(ctx, "cache too large for the in-place path (more than 524288 chunks of 128 entries)");
    return launch_compact_attn_inplace(ctx, view_mut_of(c), keep, kept, view_mut_of(spare), (const uint16_t*)q, layer_begin,
                                       layer_end, softmax_scale, out, lse, (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_append(kvtrim_ctx* ctx, kvtrim_cache* c, const void* k_new, const void* v_new,
                            const float* log_beta_new, const float* log_tail_new, const int32_t* pos_new,
                            int32_t n_new, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, c, true)) return invalid(ctx, p);
    if (!k_new || !v_new || !log_beta_new || !pos_new) return invalid(ctx, "a new-token pointer is NULL");
    if ((((uintptr_t)k_new) | ((uintptr_t)v_new)) & 15) return invalid(ctx, "k_new / v_new not 16-byte aligned");
    if (n_new < 1) return invalid(ctx, "n_new < 1");
    if ((c->log_tail == nullptr) != (log_tail_new == nullptr))
        return invalid(ctx, "log_tail_new is required exactly when the cache carries log_tail");
    return launch_append(ctx, view_mut_of(c), (const uint16_t*)k_new, (const uint16_t*)v_new, log_beta_new,
                         log_tail_new, pos_new, n_new, true, nullptr, (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_decode_step(kvtrim_ctx* ctx, kvtrim_cache* src, const void* k_new, const void* v_new,
                                 const float* log_beta_new, const float* log_tail_new, const int32_t* pos_new,
                                 int32_t n_new, const int32_t* now, const int64_t* budget, float* score_out,
                                 uint8_t* keep_out, int32_t* kept_out, uint32_t* thr_key_out, kvtrim_cache* dst,
                                 int32_t reserve, const void* q, int32_t layer_begin, int32_t layer_end,
                                 float softmax_scale, float* out, float* lse, int64_t evict_hint, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, src, true)) return invalid(ctx, p);
    if (const char* p = cache_problem(ctx, dst, true)) return invalid(ctx, p);
    if (!k_new || !v_new || !log_beta_new || !pos_new) return invalid(ctx, "a new-token pointer is NULL");
    if ((((uintptr_t)k_new) | ((uintptr_t)v_new)) & 15) return invalid(ctx, "k_new / v_new not 16-byte aligned");
    if (n_new < 1) return invalid(ctx, "n_new < 1");
    if ((src->log_tail == nullptr) != (log_tail_new == nullptr))
        return invalid(ctx, "log_tail_new is required exactly when the cache carries log_tail");
    if (!now || !budget || !score_out || !keep_out || !kept_out)
        return invalid(ctx, "now / budget / score_out / keep_out / kept_out is NULL");
    if (reserve < 0) return invalid(ctx, "reserve < 0");
    if (src->k == dst->k || src->v == dst->v || src->log_beta == dst->log_beta || src->pos == dst->pos ||
        src->seg_start == dst->seg_start || src->seg_len == dst->seg_len)
        return invalid(ctx, "src and dst share a buffer");
    if ((src->log_tail == nullptr) != (dst->log_tail == nullptr) || (src->log_tail && src->log_tail == dst->log_tail))
        return invalid(ctx, "log_tail must be set in both caches or in neither, and not shared");
    if (!q || !out) return invalid(ctx, "q / out is NULL");
    if (((uintptr_t)q) & 15) return invalid(ctx, "q not 16-byte aligned");
    if (layer_begin < 0 || layer_end > ctx->cfg.n_layers || layer_begin >= layer_end)
        return invalid(ctx, "empty or out-of-range layer range");
    if (!(softmax_scale == softmax_scale)) return invalid(ctx, "softmax_scale is NaN");
    StepArgs sa{};
    sa.k_new = (const uint16_t*)k_new;
    sa.v_new = (const uint16_t*)v_new;
    sa.lb_new = log_beta_new;
    sa.lt_new = log_tail_new;
    sa.pos_new = pos_new;
    sa.n_new = n_new;
    sa.src = view_mut_of(src);
    sa.dst = view_mut_of(dst);
    sa.reserve = reserve;
    sa.keep_out = keep_out;
    return launch_decode_step(ctx, sa.src, sa, now, budget, score_out, kept_out, thr_key_out, (const uint16_t*)q, layer_begin,
                              layer_end, softmax_scale, out, lse, evict_hint, (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_decode_step_inplace(kvtrim_ctx* ctx, kvtrim_cache* c, const void* k_new, const void* v_new,
                                         const float* log_beta_new, const float* log_tail_new, const int32_t* pos_new,
                                         int32_t n_new, const int32_t* now, const int64_t* budget, float* score_out,
                                         uint8_t* keep_out, int32_t* kept_out, uint32_t* thr_key_out, kvtrim_cache* spare,
                                         const void* q, int32_t layer_begin, int32_t layer_end, float softmax_scale,
                                         float* out, float* lse, int64_t evict_hint, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (!now || !budget || !score_out || !keep_out || !kept_out)
        return invalid(ctx, "now / budget / score_out / keep_out / kept_out is NULL");
    if (const char* p = inplace_problem(ctx, c, keep_out, kept_out, spare)) return invalid(ctx, p);
    if (!k_new || !v_new || !log_beta_new || !pos_new) return invalid(ctx, "a new-token pointer is NULL");
    if ((((uintptr_t)k_new) | ((uintptr_t)v_new)) & 15) return invalid(ctx, "k_new / v_new not 16-byte aligned");
    if (n_new < 1) return invalid(ctx, "n_new < 1");
    if ((c->log_tail == nullptr) != (log_tail_new == nullptr))
        return invalid(ctx, "log_tail_new is required exactly when the cache carries log_tail");
    if (!q || !out) return invalid(ctx, "q / out is NULL");
    if (((uintptr_t)q) & 15) return invalid(ctx, "q not 16-byte aligned");
    if (layer_begin < 0 || layer_end > ctx->cfg.n_layers || layer_begin >= layer_end)
        return invalid(ctx, "empty or out-of-range layer range");
    if (!(softmax_scale == softmax_scale)) return invalid(ctx, "softmax_scale is NaN");
    if (c->cap_entries / CMP_CHUNK + ctx->shape.nseg > ctx->ws.max_att_chunks)
        return invalid(ctx, "cache too large for the in-place path (more than 524288 chunks of 128 entries)");
    StepArgs sa{};
    sa.k_new = (const uint16_t*)k_new;
    sa.v_new = (const uint16_t*)v_new;
    sa.lb_new = log_beta_new;
    sa.lt_new = log_tail_new;
    sa.pos_new = pos_new;
    sa.n_new = n_new;
    sa.src = view_mut_of(c);
    sa.dst = view_mut_of(c);
    sa.reserve = 0;
    sa.keep_out = keep_out;
    sa.inplace = true;
    return launch_decode_step_inplace(ctx, sa.src, sa, view_mut_of(spare), now, budget, score_out, kept_out, thr_key_out,
                                      (const uint16_t*)q, layer_begin, layer_end, softmax_scale, out, lse, evict_hint,
                                      (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_append_compact(kvtrim_ctx* ctx, kvtrim_cache* src, const void* k_new, const void* v_new,
                                    const float* log_beta_new, const float* log_tail_new, const int32_t* pos_new,
                                    int32_t n_new, const int32_t* now, const int64_t* budget, float* score_out,
                                    uint8_t* keep_out, int32_t* kept_out, uint32_t* thr_key_out, kvtrim_cache* dst,
                                    int32_t reserve, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = cache_problem(ctx, src, true)) return invalid(ctx, p);
    if (const char* p = cache_problem(ctx, dst, true)) return invalid(ctx, p);
    if (!k_new || !v_new || !log_beta_new || !pos_new) return invalid(ctx, "a new-token pointer is NULL");
    if ((((uintptr_t)k_new) | ((uintptr_t)v_new)) & 15) return invalid(ctx, "k_new / v_new not 16-byte aligned");
    if (n_new < 1) return invalid(ctx, "n_new < 1");
    if ((src->log_tail == nullptr) != (log_tail_new == nullptr))
        return invalid(ctx, "log_tail_new is required exactly when the cache carries log_tail");
    if (!now || !budget || !score_out || !keep_out || !kept_out)
        return invalid(ctx, "now / budget / score_out / keep_out / kept_out is NULL");
    if (reserve < 0) return invalid(ctx, "reserve < 0");
    if (src->k == dst->k || src->v == dst->v || src->log_beta == dst->log_beta || src->pos == dst->pos ||
        src->seg_start == dst->seg_start || src->seg_len == dst->seg_len)
        return invalid(ctx, "src and dst share a buffer");
    if ((src->log_tail == nullptr) != (dst->log_tail == nullptr) || (src->log_tail && src->log_tail == dst->log_tail))
        return invalid(ctx, "log_tail must be set in both caches or in neither, and not shared");
    hipStream_t st = (hipStream_t)hip_stream;
    kvtrim_status rc = launch_append(ctx, view_mut_of(src), (const uint16_t*)k_new, (const uint16_t*)v_new, log_beta_new,
                                     log_tail_new, pos_new, n_new, false, ctx->ws.chunk_old_len, st);
    if (rc != KVTRIM_OK) return rc;
    const CacheView sv = view_of(src);
    rc = launch_score_select_general(ctx, sv, now, budget, score_out, keep_out, kept_out, thr_key_out, st);
    if (rc != KVTRIM_OK) return rc;
    launch_cmp_scan(ctx, sv, keep_out, kept_out, view_mut_of(dst), reserve, st);
    return launch_cmp_copy_new(ctx, sv, keep_out, view_mut_of(dst), (const uint16_t*)k_new, (const uint16_t*)v_new, n_new,
                               ctx->ws.chunk_old_len, st);
}

}  // extern "C"
