// C ABI of libmk.so: argument checks, HIP runtime glue, kernel launches.
// All device work is in mk_kernels.hip (included here so that the kernels and
// their launches live in one translation unit); the offline synthesis is in
// mk_sched.cpp and touches no GPU.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "mk_kernels.hip"
#include "mk_sched.h"

namespace mk {
const char *last_error_text();
}

namespace {

int hip_fail(hipError_t e, const char *what)
{
    char buf[256];
    snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(e));
    mk::set_error(buf);
    return MK_EHIP;
}
#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return hip_fail(e_, #expr); \
    } while (0)

// The kernel that walks the lists of a schedule: one per GEMV family and step count, plus the ring
// form (any step count, bf16 only).
typedef void (*walk_fn)(const mk::Params, const mk::LdsPlan);
walk_fn walk_kernel(const mk_schedule *s, int n_steps)
{
    if (s->tl.ring_pages) return mk_megakernel_ring;
    const bool multi = n_steps > 1;
    if (s->dm.w4 && s->tl.mfma) return multi ? mk_megakernel_steps_w4m : mk_megakernel_w4m;
    if (s->dm.w4) return multi ? mk_megakernel_steps_w4 : mk_megakernel_w4;
    if (s->tl.mfma) return multi ? mk_megakernel_steps_mfma : mk_megakernel_mfma;
    return multi ? mk_megakernel_steps : mk_megakernel;
}
walk_fn op_kernel(const mk_schedule *s)
{
    if (s->dm.w4) return s->tl.mfma ? mk_op_kernel_w4m : mk_op_kernel_w4;
    return s->tl.mfma ? mk_op_kernel_mfma : mk_op_kernel;
}
std::vector<const void *> all_walk_kernels()
{
    return {(const void *)mk_megakernel, (const void *)mk_megakernel_steps, (const void *)mk_op_kernel,
            (const void *)mk_megakernel_mfma, (const void *)mk_megakernel_steps_mfma, (const void *)mk_op_kernel_mfma,
            (const void *)mk_megakernel_w4, (const void *)mk_megakernel_steps_w4, (const void *)mk_op_kernel_w4,
            (const void *)mk_megakernel_w4m, (const void *)mk_megakernel_steps_w4m, (const void *)mk_op_kernel_w4m,
            (const void *)mk_megakernel_ring};
}

// ---- scratch of the allocation-free entry point -------------------------------------------------
// One array per GPU, held until the process ends.  `mk_static_scratch` names the array in device
// code only; host code uses the address hipGetSymbolAddress returns for the device that is current.
constexpr size_t kStaticScratchBytes = 16u << 20;
static __device__ __align__(256) unsigned char mk_static_scratch[kStaticScratchBytes];

struct StaticScratch {
    char *ptr = nullptr;      // device address of this GPU's copy of the array
    uint64_t owner = 0;       // serial of the schedule whose counters the array holds (0: none)
};
constexpr int kMaxDevices = 64;
StaticScratch g_static[kMaxDevices];
std::atomic<uint64_t> g_serial{0};

// Scratch regions of a schedule laid out from offset 0 of a private buffer (the workspace keeps them
// interleaved with its other regions).
struct ScratchPlan {
    uint64_t act, counters, err, tokens, total;
};
ScratchPlan plan_scratch(const mk_schedule *s)
{
    auto up = [](uint64_t v) { return (v + 4095u) / 4096u * 4096u; };
    ScratchPlan p;
    p.act = 0;
    p.counters = up(s->am.n_floats * 4);
    p.err = p.counters + up((uint64_t)s->n_counters * mk::kCounterDwords * 4);
    p.tokens = p.err + 4096;
    p.total = p.tokens + 4096;
    return p;
}

mk::Params make_params(const mk_schedule *s, const int32_t *tokens, const int32_t *positions, void *kv,
                       float *logits, int batch, int32_t *next_tokens = nullptr, int n_steps = 1, char *scratch = nullptr)
{
    mk::Params P{};
    P.ws = s->ws; P.scr = s->ws; P.lay = s->lay;
    if (scratch) {   // the scratch regions live in a buffer of their own
        const ScratchPlan sp = plan_scratch(s);
        P.scr = scratch;
        P.lay.act = sp.act; P.lay.counters = sp.counters; P.lay.err = sp.err; P.lay.tokens = sp.tokens;
    }
    P.tokens = tokens; P.positions = positions; P.kv = (uint16_t *)kv; P.logits = logits;
    P.next_tokens = next_tokens ? next_tokens : (int32_t *)(P.scr + P.lay.tokens);
    P.n_steps = n_steps; P.amax = s->am.amax; P.want_tokens = next_tokens != nullptr;
    P.batch = batch; P.max_batch = s->dm.Bm; P.max_context = s->dm.Tm;
    P.n_layers = s->dm.L; P.hidden = s->dm.H; P.n_q_heads = s->dm.nq; P.n_kv_heads = s->dm.nkv;
    P.head_dim = s->dm.d; P.inter_pad = s->gm.ipad; P.vocab = s->dm.V;
    P.qk_norm = s->cfg.qk_norm; P.rms_eps = s->cfg.rms_eps;
    P.epoch = s->epoch; P.spin_limit = s->cfg.spin_limit ? s->cfg.spin_limit : (1u << 20);
    P.max_instr = (uint32_t)s->max_instr; P.flags = s->cfg.flags;
    P.embed_chunk = s->wm.embed; P.embed_kbt = (uint32_t)s->gm.head.kbt; P.embed_rlog = (uint32_t)s->gm.head.rlog;
    P.only_seq = mk::kNone; P.act_bytes = (uint32_t)(s->am.n_floats * 4);
    P.w4_group = s->dm.w4 ? (uint32_t)s->dm.group : 0u;
    return P;
}

int check_step_args(mk_schedule *s, const int32_t *tokens, const int32_t *positions, void *kv, float *logits, int batch)
{
    if (!s) { mk::set_error("null schedule"); return MK_EINVAL; }
    if (!s->bound) { mk::set_error("mk_decode_step before mk_bind_workspace"); return MK_ESTATE; }
    if (!s->loaded) { mk::set_error("mk_decode_step before mk_load_weights"); return MK_ESTATE; }
    if (!tokens || !positions || !kv || !logits) { mk::set_error("null device pointer"); return MK_EINVAL; }
    if (batch < 1 || batch > s->dm.Bm) { mk::set_error("batch outside 1..max_batch"); return MK_EINVAL; }
    return MK_OK;
}

int fill_u32(void *dst, uint32_t v, size_t n, hipStream_t st)
{
    if (!n) return MK_OK;
    hipLaunchKernelGGL(mk_fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (uint32_t *)dst, v, n);
    HIP_TRY(hipGetLastError());
    return MK_OK;
}

int reset_sync_state(mk_schedule *s, hipStream_t st)
{
    int rc = fill_u32(s->ws + s->lay.counters, 0u, (size_t)s->n_counters * mk::kCounterDwords, st);
    if (rc) return rc;
    rc = fill_u32(s->ws + s->lay.err, 0u, 16, st);
    s->epoch = 0;
    return rc;
}

}  // namespace

extern "C" {

const char *mk_last_error(void) { return mk::last_error_text(); }

int64_t mk_pages_available(int64_t a, int64_t b, int64_t c, int64_t d, int64_t e, int64_t f) { return mk::pages_available(a, b, c, d, e, f); }
int64_t mk_pipeline_stages(int64_t a, int64_t b, int64_t c, int64_t d, int64_t e) { return mk::pipeline_stages(a, b, c, d, e); }

int mk_build_schedule(const mk_config *cfg, mk_schedule **out)
{
    if (!cfg || !out) { mk::set_error("null argument"); return MK_EINVAL; }
    mk_config c = *cfg;
    if (c.n_workgroups == 0) {
        hipDeviceProp_t prop;
        HIP_TRY(hipGetDeviceProperties(&prop, c.device_id));
        c.n_workgroups = prop.multiProcessorCount;
    }
    try {
        return mk::build_schedule(&c, out);
    } catch (const std::exception &e) {
        mk::set_error(std::string("mk_build_schedule: ") + e.what());
        return MK_ENOMEM;
    }
}

int mk_schedule_verify(const mk_schedule *s)
{
    try { return mk::verify_schedule(s); }
    catch (const std::exception &e) { mk::set_error(std::string("mk_schedule_verify: ") + e.what()); return MK_ENOMEM; }
}

int mk_schedule_dump(const mk_schedule *s, void *buf, size_t *bytes) { return mk::dump_schedule(s, buf, bytes); }

int mk_schedule_load(const void *buf, size_t bytes, mk_schedule **out)
{
    try { return mk::load_schedule(buf, bytes, out); }
    catch (const std::exception &e) { mk::set_error(std::string("mk_schedule_load: ") + e.what()); return MK_ENOMEM; }
}

int mk_get_config(const mk_schedule *s, mk_config *out)
{
    if (!s || !out) { mk::set_error("null argument"); return MK_EINVAL; }
    *out = s->cfg;
    return MK_OK;
}

int mk_get_stats(const mk_schedule *s, mk_stats *o)
{
    if (!s || !o) { mk::set_error("null argument"); return MK_EINVAL; }
    memset(o, 0, sizeof *o);
    o->n_workgroups = s->n_wg; o->threads_per_wg = mk::kWgThreads; o->n_tasks = s->n_tasks; o->n_counters = s->n_counters;
    o->max_instr_per_wg = s->max_instr - 1;
    o->split_qkv = s->tl.s_qkv; o->split_o = s->tl.s_o; o->split_gateup = s->tl.s_gu; o->split_down = s->tl.s_d;
    o->attn_chunks = s->tl.nc; o->use_mfma = s->tl.mfma;
    o->lds_bytes = (int32_t)s->lds_total; o->ring_pages = s->tl.ring_pages; o->page_bytes = s->tl.page_bytes; o->n_stage = s->tl.n_stage;
    const mk::Dims &d = s->dm;
    const mk::Geom &g = s->gm;
    auto chunks = [](const mk::MatGeom &m) { return (int64_t)m.groups * m.kbt; };
    int64_t per_layer = chunks(g.qkv) + chunks(g.o) + chunks(g.gu) + chunks(g.down);
    o->weight_bytes_per_step = (per_layer * d.L + chunks(g.head)) * mk::kChunkBytes +
                               (d.w4 ? per_layer * d.L * (2048 / d.group) * 2 : 0);
    o->rows_qkv = g.qkv.R; o->rows_o = g.o.R; o->rows_gateup = g.gu.R; o->rows_down = g.down.R; o->rows_head = g.head.R;
    o->workspace_bytes = (int64_t)s->lay.total;
    o->sim_makespan_us = s->sim.makespan_us; o->sim_duty_cycle = s->sim.duty;
    o->candidates_tried = s->cand_tried; o->candidates_pruned = s->cand_pruned;
    o->fuse_combine = s->tl.fuse;
    o->from_table = s->from_table;
    o->attention_mfma = s->tl.att_mc;
    return MK_OK;
}

int mk_instr_count(const mk_schedule *s, int32_t wg)
{
    if (!s || wg < 0 || wg >= s->n_wg) { mk::set_error("bad workgroup index"); return MK_EINVAL; }
    const mk::Instr *l = (const mk::Instr *)s->instr.data() + (size_t)wg * s->max_instr;
    int n = 0;
    while (n < s->max_instr && l[n].op != mk::OP_END) ++n;
    return n;
}

int mk_instr_get(const mk_schedule *s, int32_t wg, int32_t idx, uint32_t *out32)
{
    if (!s || !out32 || wg < 0 || wg >= s->n_wg || idx < 0 || idx >= s->max_instr) { mk::set_error("bad instruction index"); return MK_EINVAL; }
    memcpy(out32, s->instr.data() + ((size_t)wg * s->max_instr + idx) * mk::kInstrDwords, mk::kInstrDwords * 4);
    return MK_OK;
}

int mk_instr_set(mk_schedule *s, int32_t wg, int32_t idx, const uint32_t *in32)
{
    if (!s || !in32 || wg < 0 || wg >= s->n_wg || idx < 0 || idx >= s->max_instr) { mk::set_error("bad instruction index"); return MK_EINVAL; }
    if (s->bound) { mk::set_error("instructions are frozen once the workspace is bound"); return MK_ESTATE; }
    memcpy(s->instr.data() + ((size_t)wg * s->max_instr + idx) * mk::kInstrDwords, in32, mk::kInstrDwords * 4);
    return MK_OK;
}

size_t mk_workspace_bytes(const mk_schedule *s) { return s ? (size_t)s->lay.total : 0; }

int mk_bind_workspace(mk_schedule *s, void *dev, size_t bytes, void *stream)
{
    if (!s || !dev) { mk::set_error("null argument"); return MK_EINVAL; }
    if (bytes < s->lay.total) { mk::set_error("workspace smaller than mk_workspace_bytes()"); return MK_ENOMEM; }
    if (((uintptr_t)dev & 255u) != 0) { mk::set_error("workspace must be 256-byte aligned"); return MK_EINVAL; }
    if (mk::verify_schedule(s) != MK_OK) return MK_ESCHED;
    hipStream_t st = (hipStream_t)stream;
    hipPointerAttribute_t attr;
    HIP_TRY(hipPointerGetAttributes(&attr, dev));
    if (attr.type != hipMemoryTypeDevice) { mk::set_error("workspace is not device memory"); return MK_EINVAL; }
    s->device = attr.device;
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, s->device));
    if (std::string(prop.gcnArchName).rfind("gfx950", 0) != 0) { mk::set_error(std::string("device is ") + prop.gcnArchName + ", this library is built for gfx950"); return MK_EHIP; }
    for (const void *k : all_walk_kernels())
        HIP_TRY(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)s->lds_total));
    // every kernel this handle can launch spins on dependency counters (or is launched with the same grid):
    // all of its workgroups must be resident at once
    for (const void *k : {(const void *)walk_kernel(s, 1), (const void *)walk_kernel(s, 2), (const void *)op_kernel(s)}) {
        int per_cu = 0;
        HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k, mk::kWgThreads, s->lds_total));
        if ((int64_t)per_cu * prop.multiProcessorCount < s->n_wg) {
            char buf[200];
            snprintf(buf, sizeof buf, "the device keeps only %d x %d workgroups resident, the schedule needs %d", per_cu, prop.multiProcessorCount, s->n_wg);
            mk::set_error(buf);
            return MK_EINFEASIBLE;
        }
    }
    s->ws = (char *)dev; s->ws_bytes = bytes;
    // instruction lists
    HIP_TRY(hipMemcpyAsync(s->ws + s->lay.instr, s->instr.data(), s->instr.size() * 4, hipMemcpyHostToDevice, st));
    // weight stream of every workgroup: (first chunk, chunk count) of its GEMV tasks in list order
    std::vector<uint32_t> wstream((size_t)s->n_wg * s->max_instr * 2, mk::kNone);
    for (int w = 0; w < s->n_wg; ++w) {
        const mk::Instr *l = (const mk::Instr *)s->instr.data() + (size_t)w * s->max_instr;
        uint32_t *dst = wstream.data() + (size_t)w * s->max_instr * 2;
        for (int i = 0, e = 0; i < s->max_instr && l[i].op != mk::OP_END; ++i) {
            if (l[i].op != mk::OP_GEMV) continue;
            const mk::Instr &I = l[i];
            if (I.S == 0) { mk::set_error("a GEMV task has zero K splits"); return MK_ESCHED; }
            const bool sm = (I.flags & mk::F_SLICE_MAJOR) != 0;
            const uint32_t groups = mk::instr_groups(I);
            const uint32_t first = mk::unit_chunk0(sm, I.u0, I.S, groups, I.kbt, I.nkb);
            const uint32_t total = mk::unit_chunk0(sm, I.u0 + I.nu, I.S, groups, I.kbt, I.nkb) - first;
            if ((uint64_t)I.w_chunk + first + total > s->wm.n_chunks) { mk::set_error("a GEMV task reaches beyond the weight region"); return MK_ESCHED; }
            dst[2 * e] = I.w_chunk + first; dst[2 * e + 1] = total;
            ++e;
        }
    }
    HIP_TRY(hipMemcpyAsync(s->ws + s->lay.stream, wstream.data(), wstream.size() * 4, hipMemcpyHostToDevice, st));
    // RoPE table: angle = pos * theta^(-2i/d), evaluated in double, stored as (cos, sin) fp32
    {
        const int d = s->dm.d, T = s->dm.Tm;
        std::vector<float> tab((size_t)T * d);
        std::vector<double> freq(d / 2);
        for (int i = 0; i < d / 2; ++i) freq[i] = std::pow((double)s->cfg.rope_theta, -2.0 * i / d);
        for (int p = 0; p < T; ++p)
            for (int i = 0; i < d / 2; ++i) {
                double ang = (double)p * freq[i];
                tab[((size_t)p * (d / 2) + i) * 2] = (float)std::cos(ang);
                tab[((size_t)p * (d / 2) + i) * 2 + 1] = (float)std::sin(ang);
            }
        HIP_TRY(hipMemcpyAsync(s->ws + s->lay.rope, tab.data(), tab.size() * 4, hipMemcpyHostToDevice, st));
        HIP_TRY(hipStreamSynchronize(st));   // the host vectors above (and the stream table) die here
    }
    int rc = reset_sync_state(s, st);
    if (rc) return rc;
    if (s->cfg.flags & MK_F_TRACE) {
        rc = fill_u32(s->ws + s->lay.trace, 0u, (size_t)s->n_wg * s->max_instr * 16, st);
        if (rc) return rc;
    }
    if (!s->ev_valid) {
        hipEvent_t a, b;
        HIP_TRY(hipEventCreate(&a));
        HIP_TRY(hipEventCreate(&b));
        s->ev0 = a; s->ev1 = b; s->ev_valid = true;
    }
    s->bound = true; s->loaded = false;
    return MK_OK;
}

static int repack(const void *src, int n_rows, int n_cols, mk_schedule *s, uint32_t chunk0, const mk::MatGeom &m,
                  uint32_t rpu, uint32_t r_off, uint32_t g0, uint32_t n_groups, hipStream_t st, const void *scales = nullptr)
{
    if (!src) { mk::set_error("mk_load_weights: a required matrix pointer is NULL"); return MK_EINVAL; }
    size_t total = (size_t)n_groups * m.kbt * 64;
    mk::u32x4 *dst = (mk::u32x4 *)(s->ws + s->lay.weights) + (size_t)chunk0 * 64;
    const mk::ChunkOrder ord = {(uint32_t)m.S, (uint32_t)((m.kbt + m.S - 1) / m.S), (uint32_t)m.groups, (uint32_t)m.sm};
    if (m.w4) {
        if (!scales) { mk::set_error("mk_load_weights: weight_bits is 4 but a scale pointer is NULL"); return MK_EINVAL; }
        hipLaunchKernelGGL(mk_repack_w4_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const uint8_t *)src,
                           n_rows, n_cols, dst, (uint32_t)m.kbt, (uint32_t)m.rlog, rpu, r_off, g0, n_groups, (uint32_t)(s->tl.mfma ? 1 : 0), ord);
        HIP_TRY(hipGetLastError());
        const uint32_t spc = 2048u / (uint32_t)s->dm.group;
        const size_t n_s = (size_t)n_groups * m.kbt * spc;
        uint16_t *sdst = (uint16_t *)(s->ws + s->lay.wscale) + (size_t)chunk0 * spc;
        hipLaunchKernelGGL(mk_repack_scales_kernel, dim3((unsigned)((n_s + 255) / 256)), dim3(256), 0, st,
                           (const uint16_t *)scales, n_rows, n_cols, sdst, (uint32_t)m.kbt, (uint32_t)m.rlog, rpu, r_off, g0,
                           n_groups, (uint32_t)s->dm.group, ord);
        HIP_TRY(hipGetLastError());
        return MK_OK;
    }
    hipLaunchKernelGGL(mk_repack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const uint16_t *)src, n_rows,
                       n_cols, dst, (uint32_t)m.kbt, (uint32_t)m.rlog, rpu, r_off, g0, n_groups, ord);
    HIP_TRY(hipGetLastError());
    return MK_OK;
}

static int copy_vec(const void *src, size_t n, char *ws, uint64_t vbase, uint32_t off, hipStream_t st)
{
    if (!src) { mk::set_error("mk_load_weights: a required vector pointer is NULL"); return MK_EINVAL; }
    hipLaunchKernelGGL(mk_copy_u16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const uint16_t *)src,
                       (uint16_t *)(ws + vbase) + off, n);
    HIP_TRY(hipGetLastError());
    return MK_OK;
}

int mk_load_weights(mk_schedule *s, const mk_weights *w, void *stream)
{
    if (!s || !w) { mk::set_error("null argument"); return MK_EINVAL; }
    if (!s->bound) { mk::set_error("mk_load_weights before mk_bind_workspace"); return MK_ESTATE; }
    hipStream_t st = (hipStream_t)stream;
    const mk::Dims &d = s->dm;
    const mk::WeightMap &m = s->wm;
    char *ws = s->ws;
    const uint64_t vb = s->lay.vecs;
    if (!w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->mlp_norm || !w->w_gate || !w->w_up || !w->w_down) {
        mk::set_error("mk_load_weights: a per-layer pointer table is NULL");
        return MK_EINVAL;
    }
    if (s->cfg.qkv_bias && (!w->bq || !w->bk || !w->bv)) { mk::set_error("mk_load_weights: qkv_bias set but a bias table is NULL"); return MK_EINVAL; }
    if (s->cfg.qk_norm && (!w->q_norm || !w->k_norm)) { mk::set_error("mk_load_weights: qk_norm set but a gain table is NULL"); return MK_EINVAL; }
    const bool w4 = s->dm.w4 != 0;
    if (w4 && (!w->sq || !w->sk || !w->sv || !w->so || !w->s_gate || !w->s_up || !w->s_down)) {
        mk::set_error("mk_load_weights: weight_bits is 4 but a scale table is NULL");
        return MK_EINVAL;
    }
    auto sc = [&](const void *const *tab, int l) -> const void * { return w4 ? tab[l] : nullptr; };
    int rc;
#define TRY(x) do { rc = (x); if (rc) return rc; } while (0)
    const mk::Geom &g = s->gm;
    for (int l = 0; l < d.L; ++l) {
        const uint32_t R = (uint32_t)g.qkv.R;
        TRY(repack(w->wq[l], d.qd, d.H, s, m.qkv[l], g.qkv, R, 0, 0, d.qd / R, st, sc(w->sq, l)));
        TRY(repack(w->wk[l], d.kvd, d.H, s, m.qkv[l], g.qkv, R, 0, d.qd / R, d.kvd / R, st, sc(w->sk, l)));
        TRY(repack(w->wv[l], d.kvd, d.H, s, m.qkv[l], g.qkv, R, 0, (d.qd + d.kvd) / R, d.kvd / R, st, sc(w->sv, l)));
        TRY(repack(w->wo[l], d.H, d.qd, s, m.o[l], g.o, (uint32_t)g.o.R, 0, 0, (uint32_t)g.o.groups, st, sc(w->so, l)));
        // gate rows fill the lower half of every row group, up rows the upper half
        const uint32_t half = (uint32_t)g.gu.R / 2;
        TRY(repack(w->w_gate[l], d.I, d.H, s, m.gu[l], g.gu, half, 0, 0, (uint32_t)g.gu.groups, st, sc(w->s_gate, l)));
        TRY(repack(w->w_up[l], d.I, d.H, s, m.gu[l], g.gu, half, half, 0, (uint32_t)g.gu.groups, st, sc(w->s_up, l)));
        TRY(repack(w->w_down[l], d.H, d.I, s, m.down[l], g.down, (uint32_t)g.down.R, 0, 0, (uint32_t)g.down.groups, st, sc(w->s_down, l)));
        TRY(copy_vec(w->attn_norm[l], d.H, ws, vb, m.g_attn[l], st));
        TRY(copy_vec(w->mlp_norm[l], d.H, ws, vb, m.g_mlp[l], st));
        if (s->cfg.qkv_bias) {
            TRY(copy_vec(w->bq[l], d.qd, ws, vb, m.bias[l], st));
            TRY(copy_vec(w->bk[l], d.kvd, ws, vb, m.bias[l] + d.qd, st));
            TRY(copy_vec(w->bv[l], d.kvd, ws, vb, m.bias[l] + d.qd + d.kvd, st));
        }
        if (s->cfg.qk_norm) {
            TRY(copy_vec(w->q_norm[l], d.d, ws, vb, m.qn[l], st));
            TRY(copy_vec(w->k_norm[l], d.d, ws, vb, m.kn[l], st));
        }
    }
    TRY(repack(w->embed, d.V, d.H, s, m.embed, g.head, (uint32_t)g.head.R, 0, 0, (uint32_t)g.head.groups, st));
    if (!s->cfg.tie_embeddings) TRY(repack(w->lm_head, d.V, d.H, s, m.head, g.head, (uint32_t)g.head.R, 0, 0, (uint32_t)g.head.groups, st));
    TRY(copy_vec(w->final_norm, d.H, ws, vb, m.g_final, st));
#undef TRY
    s->loaded = true;
    return MK_OK;
}

static int launch_steps(mk_schedule *s, const int32_t *tokens, const int32_t *positions, void *kv, float *logits,
                        int32_t *next_tokens, int32_t batch, int32_t n_steps, hipStream_t st)
{
    if ((uint64_t)s->epoch + (uint64_t)n_steps >= 0x00800000u) {   // keep epoch * signals far from wrapping
        int rc = reset_sync_state(s, st);
        if (rc) return rc;
    }
    mk::Params P = make_params(s, tokens, positions, kv, logits, batch, next_tokens, n_steps);
    s->last_static = false;
    P.epoch = s->epoch + 1;
    s->epoch += (uint32_t)n_steps;
    mk::LdsPlan lp{s->lds_red_bytes, s->lds_xs_off, s->lds_ring_off, s->lds_ring_slots};
    const bool timing = (s->cfg.flags & MK_F_TIMING) != 0;
    if (timing) HIP_TRY(hipEventRecord((hipEvent_t)s->ev0, st));
    hipLaunchKernelGGL(walk_kernel(s, n_steps), dim3((unsigned)s->n_wg), dim3(mk::kWgThreads), s->lds_total, st, P, lp);
    HIP_TRY(hipGetLastError());
    if (timing) HIP_TRY(hipEventRecord((hipEvent_t)s->ev1, st));
    return MK_OK;
}

int mk_decode_step(mk_schedule *s, const int32_t *tokens, const int32_t *positions, void *kv, float *logits,
                   int32_t batch, void *stream)
{
    int rc = check_step_args(s, tokens, positions, kv, logits, batch);
    if (rc) return rc;
    return launch_steps(s, tokens, positions, kv, logits, nullptr, batch, 1, (hipStream_t)stream);
}

int mk_decode_steps(mk_schedule *s, const int32_t *tokens, const int32_t *positions, void *kv, float *logits,
                    int32_t *tokens_out, int32_t batch, int32_t n_steps, void *stream)
{
    int rc = check_step_args(s, tokens, positions, kv, logits, batch);
    if (rc) return rc;
    if (!tokens_out) { mk::set_error("null device pointer"); return MK_EINVAL; }
    if (n_steps < 1 || n_steps > s->dm.Tm) { mk::set_error("n_steps outside 1..max_context"); return MK_EINVAL; }
    return launch_steps(s, tokens, positions, kv, logits, tokens_out, batch, n_steps, (hipStream_t)stream);
}

int mk_fill_cache(mk_schedule *s, const int32_t *tokens, const int32_t *positions, void *kv, int32_t batch, int32_t n_tokens,
                  void *stream)
{
    if (!s) { mk::set_error("null schedule"); return MK_EINVAL; }
    if (!s->bound) { mk::set_error("mk_fill_cache before mk_bind_workspace"); return MK_ESTATE; }
    if (!s->loaded) { mk::set_error("mk_fill_cache before mk_load_weights"); return MK_ESTATE; }
    if (!tokens || !positions || !kv) { mk::set_error("null device pointer"); return MK_EINVAL; }
    if (batch < 1 || batch > s->dm.Bm) { mk::set_error("batch outside 1..max_batch"); return MK_EINVAL; }
    if (n_tokens < 1 || n_tokens > s->dm.Tm) { mk::set_error("n_tokens outside 1..max_context"); return MK_EINVAL; }
    hipStream_t st = (hipStream_t)stream;
    if ((uint64_t)s->epoch + (uint64_t)n_tokens >= 0x00800000u) {   // keep epoch * signals far from wrapping
        int rc = reset_sync_state(s, st);
        if (rc) return rc;
    }
    mk::Params P = make_params(s, tokens, positions, kv, nullptr, batch, nullptr, n_tokens);
    P.forced_tokens = tokens;
    s->last_static = false;
    P.epoch = s->epoch + 1;
    s->epoch += (uint32_t)n_tokens;
    mk::LdsPlan lp{s->lds_red_bytes, s->lds_xs_off, s->lds_ring_off, s->lds_ring_slots};
    const bool timing = (s->cfg.flags & MK_F_TIMING) != 0;
    if (timing) HIP_TRY(hipEventRecord((hipEvent_t)s->ev0, st));
    // (always the kernel that walks its lists once per step, also for a single token: only it knows forced tokens)
    hipLaunchKernelGGL(walk_kernel(s, 2), dim3((unsigned)s->n_wg), dim3(mk::kWgThreads), s->lds_total, st, P, lp);
    HIP_TRY(hipGetLastError());
    if (timing) HIP_TRY(hipEventRecord((hipEvent_t)s->ev1, st));
    return MK_OK;
}

int mk_decode_step_per_op(mk_schedule *s, const int32_t *tokens, const int32_t *positions, void *kv, float *logits,
                          int32_t batch, void *stream)
{
    int rc = check_step_args(s, tokens, positions, kv, logits, batch);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    mk::Params P = make_params(s, tokens, positions, kv, logits, batch);
    s->last_static = false;
    mk::LdsPlan lp{s->lds_red_bytes, s->lds_xs_off, 0, 0};
    const bool timing = (s->cfg.flags & MK_F_TIMING) != 0;
    if (timing) HIP_TRY(hipEventRecord((hipEvent_t)s->ev0, st));
    for (uint32_t seq : s->ref_seqs) {
        P.only_seq = seq;
        hipLaunchKernelGGL(op_kernel(s), dim3((unsigned)s->n_wg), dim3(mk::kWgThreads), s->lds_total, st, P, lp);
    }
    HIP_TRY(hipGetLastError());
    if (timing) HIP_TRY(hipEventRecord((hipEvent_t)s->ev1, st));
    return MK_OK;
}

// This GPU's copy of the static scratch array (looked up once per device, with that device current).
static int static_scratch_of(int device, StaticScratch **out)
{
    if (device < 0 || device >= kMaxDevices) { mk::set_error("device index beyond the static scratch table"); return MK_EINVAL; }
    StaticScratch &st = g_static[device];
    if (!st.ptr) {
        int cur = -1;
        HIP_TRY(hipGetDevice(&cur));
        if (cur != device) HIP_TRY(hipSetDevice(device));
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(mk_static_scratch));
        if (cur != device) (void)hipSetDevice(cur);
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(mk_static_scratch)");
        if (!p) { mk::set_error("the static scratch array has no address on this device"); return MK_EHIP; }
        st.ptr = (char *)p;
    }
    *out = &st;
    return MK_OK;
}

int mk_decode_step_static(mk_schedule *s, const int32_t *tokens, const int32_t *positions, void *kv, float *logits,
                          int32_t batch, void *stream)
{
    if (!s) { mk::set_error("null schedule"); return MK_EINVAL; }
    const ScratchPlan sp = plan_scratch(s);
    if (sp.total > kStaticScratchBytes) {   // (checked first: a property of the schedule, whatever its binding state)
        char buf[200];
        snprintf(buf, sizeof buf, "mk_decode_step_static: this schedule needs %llu bytes of scratch, the static array holds %llu",
                 (unsigned long long)sp.total, (unsigned long long)kStaticScratchBytes);
        mk::set_error(buf);
        return MK_ENOMEM;
    }
    int rc = check_step_args(s, tokens, positions, kv, logits, batch);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    StaticScratch *ss = nullptr;
    rc = static_scratch_of(s->device, &ss);
    if (rc) return rc;
    if (!s->serial) s->serial = ++g_serial;
    // The step number lives in the array itself and a one-workgroup kernel advances it ahead of every step (and zeroes the
    // counters when the array holds another schedule's, or none, or the number nears the wrap range): a call recorded
    // into a graph therefore replays correctly.  Kernels, not memsets, for the same reason.
    const uint32_t reset = ss->owner != s->serial ? 1u : 0u;
    if (reset) {
        rc = fill_u32(ss->ptr + sp.err, 0u, 16, st);
        if (rc) return rc;
        ss->owner = s->serial;
    }
    uint32_t *epoch_dev = (uint32_t *)(ss->ptr + sp.tokens + 2048);
    hipLaunchKernelGGL(mk_static_begin_kernel, dim3(1), dim3(1024), 0, st, epoch_dev, (uint32_t *)(ss->ptr + sp.counters),
                       (size_t)s->n_counters * mk::kCounterDwords, reset);
    HIP_TRY(hipGetLastError());
    mk::Params P = make_params(s, tokens, positions, kv, logits, batch, nullptr, 1, ss->ptr);
    P.epoch = 0; P.epoch_ptr = epoch_dev;
    mk::LdsPlan lp{s->lds_red_bytes, s->lds_xs_off, s->lds_ring_off, s->lds_ring_slots};
    hipLaunchKernelGGL(walk_kernel(s, 1), dim3((unsigned)s->n_wg), dim3(mk::kWgThreads), s->lds_total, st, P, lp);
    HIP_TRY(hipGetLastError());
    s->last_static = true;
    return MK_OK;
}

int mk_check(mk_schedule *s, void *stream)
{
    if (!s || !s->bound) { mk::set_error("mk_check on an unbound schedule"); return MK_ESTATE; }
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipStreamSynchronize(st));
    uint32_t e[16] = {0};
    StaticScratch *ss = nullptr;
    if (s->last_static) {
        int rc0 = static_scratch_of(s->device, &ss);
        if (rc0) return rc0;
        HIP_TRY(hipMemcpy(e, ss->ptr + plan_scratch(s).err, sizeof e, hipMemcpyDeviceToHost));
    } else {
        HIP_TRY(hipMemcpy(e, s->ws + s->lay.err, sizeof e, hipMemcpyDeviceToHost));
    }
    if (e[0] == 0 && e[1] == 0 && e[2] == 0) return MK_OK;
    int rc = MK_OK;
    if (ss) ss->owner = 0;                 // the next step on the static array starts from zeroed counters and flags
    else rc = reset_sync_state(s, st);
    HIP_TRY(hipStreamSynchronize(st));
    if (rc) return rc;
    char buf[200];
    if (e[0]) {
        snprintf(buf, sizeof buf, "a dependency wait hit the spin limit (first reported at instruction %u of some workgroup)", e[0] - 1);
        mk::set_error(buf);
        return MK_ETIMEOUT;
    }
    if (e[2]) {
        mk::set_error("the weight-page ring ran dry: stream table and instruction lists disagree");
        return MK_ESCHED;
    }
    mk::set_error(e[1] == 1 ? "token id outside [0, vocab)" : "position outside [0, max_context)");
    return MK_EINVAL;
}

int mk_last_step_ms(mk_schedule *s, float *ms)
{
    if (!s || !ms || !s->ev_valid) { mk::set_error("no timed step"); return MK_ESTATE; }
    if (!(s->cfg.flags & MK_F_TIMING)) { mk::set_error("step timing needs flag bit 1 (value 2) in mk_config.flags"); return MK_ESTATE; }
    HIP_TRY(hipEventSynchronize((hipEvent_t)s->ev1));
    HIP_TRY(hipEventElapsedTime(ms, (hipEvent_t)s->ev0, (hipEvent_t)s->ev1));
    return MK_OK;
}

int mk_read_ceiling(mk_schedule *s, int32_t reps, float *ms_out, size_t *bytes, void *stream)
{
    if (!s || !ms_out || !bytes || reps < 1) { mk::set_error("bad argument"); return MK_EINVAL; }
    if (!s->bound || !s->ev_valid) { mk::set_error("mk_read_ceiling needs a bound workspace"); return MK_ESTATE; }
    hipStream_t st = (hipStream_t)stream;
    const uint64_t per_wg = s->wm.n_chunks / (uint64_t)s->n_wg;
    if (per_wg == 0 || per_wg > 0xffffffffull) { mk::set_error("weight region too small or too large to stream"); return MK_EINVAL; }
    const mk::u32x4 *src = (const mk::u32x4 *)(s->ws + s->lay.weights);
    *bytes = (size_t)(per_wg * (uint64_t)s->n_wg * mk::kChunkBytes);
    for (int r = -1; r < reps; ++r) {
        if (r >= 0) HIP_TRY(hipEventRecord((hipEvent_t)s->ev0, st));
        hipLaunchKernelGGL(mk_stream_read_kernel, dim3((unsigned)s->n_wg), dim3(mk::kWgThreads), 0, st, src, (uint32_t)per_wg,
                           (uint32_t *)(s->ws + s->lay.tokens));
        HIP_TRY(hipGetLastError());
        if (r >= 0) {
            HIP_TRY(hipEventRecord((hipEvent_t)s->ev1, st));
            HIP_TRY(hipEventSynchronize((hipEvent_t)s->ev1));
            HIP_TRY(hipEventElapsedTime(&ms_out[r], (hipEvent_t)s->ev0, (hipEvent_t)s->ev1));
        }
    }
    HIP_TRY(hipStreamSynchronize(st));
    return MK_OK;
}

int mk_set_flags(mk_schedule *s, uint32_t flags)
{
    if (!s) { mk::set_error("null schedule"); return MK_EINVAL; }
    if ((flags ^ s->cfg.flags) & ~(uint32_t)MK_F_TIMING) { mk::set_error("only MK_F_TIMING can change after the build"); return MK_EINVAL; }
    s->cfg.flags = flags;
    return MK_OK;
}

int mk_read_trace(mk_schedule *s, uint64_t *host_out, size_t *n_records, void *stream)
{
    if (!s || !host_out || !n_records || !s->bound) { mk::set_error("bad argument"); return MK_EINVAL; }
    if (!(s->cfg.flags & MK_F_TRACE)) { mk::set_error("schedule was built without MK_F_TRACE"); return MK_ESTATE; }
    size_t have = (size_t)s->n_wg * s->max_instr;
    size_t n = *n_records < have ? *n_records : have;
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    HIP_TRY(hipMemcpy(host_out, s->ws + s->lay.trace, n * 64, hipMemcpyDeviceToHost));
    *n_records = n;
    return MK_OK;
}

void mk_destroy(mk_schedule *s)
{
    if (!s) return;
    if (s->ev_valid) {
        (void)hipEventDestroy((hipEvent_t)s->ev0);
        (void)hipEventDestroy((hipEvent_t)s->ev1);
    }
    delete s;
}

}  // extern "C"
