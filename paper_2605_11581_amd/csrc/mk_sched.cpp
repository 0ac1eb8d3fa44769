// Offline synthesis of the static schedule (paper Sec. 3 Phase I).
//
//   Step 1-2 (Sec. 4.2.2): the decoder + LM head become a DAG of tile-tasks.
//     Tasks are emitted operator by operator; their dependency edges are the
//     read-after-write pairs a last-writers table finds when the tasks are
//     walked in topological (operator) order.  At run time the edges are
//     carried by global counters: a task signals its operator instance's
//     counter, a consumer waits until the counter has all of its signals.
//   Step 3 (Sec. 4.2.2) + Sec. 4.1.1: candidates (K splits per operator,
//     attention chunking, LDS page ring) are pruned by the on-chip memory
//     budget of Eq. 1-2.
//   Step 4: every surviving candidate is run through a pipeline simulator; the
//     one with the smallest makespan (ties: highest duty cycle) is serialised
//     as per-workgroup instruction lists.
#include "mk_sched.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <dlfcn.h>

#include <fstream>
#include <map>
#include <numeric>
#include <sstream>

namespace mk {

static thread_local std::string g_err;
void set_error(const std::string &msg) { g_err = msg; }
const char *last_error_text() { return g_err.c_str(); }

constexpr int64_t kLdsMax = 160 * 1024;   // LDS per CU on CDNA4
constexpr int kMaxHidden = 16 * kWgThreads;
constexpr int kPartPad = 4;   // attention partial rows: [acc[d], m, l, pad, pad]

int64_t pages_available(int64_t smem_max, int64_t n_stage, int64_t instr_buf, int64_t semaphores,
                        int64_t scratch, int64_t page_size)
{
    int64_t left = smem_max - n_stage * (instr_buf + semaphores + scratch);
    if (left < 0 || page_size <= 0) return 0;
    return left / page_size;
}

int64_t pipeline_stages(int64_t pages_total, int64_t pages_weight, int64_t pages_scale, int64_t pages_act,
                        int64_t pages_per_stage)
{
    int64_t left = pages_total - pages_weight - pages_scale - pages_act;
    if (left < 0 || pages_per_stage <= 0) return 0;
    return left / pages_per_stage;
}

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

static int derive_dims(const mk_config &c, Dims &d)
{
    char buf[256];
    auto bad = [&](const char *what) {
        snprintf(buf, sizeof buf, "mk_config: %s", what);
        set_error(buf);
        return MK_EINVAL;
    };
    if (c.n_layers < 1 || c.hidden < 32 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.intermediate < 1 || c.vocab < 1)
        return bad("non-positive dimension");
    if (c.hidden % 32 != 0) return bad("hidden must be a multiple of 32");
    if (c.hidden > kMaxHidden) return bad("hidden larger than 4096 is not supported");
    if (c.head_dim != 64 && c.head_dim != 128) return bad("head_dim must be 64 or 128");
    if (c.n_q_heads % c.n_kv_heads != 0) return bad("n_q_heads must be a multiple of n_kv_heads");
    if (c.n_q_heads / c.n_kv_heads > kMaxGroup) return bad("more than 8 q heads per kv head");
    if (c.max_batch < 1 || c.max_batch > kMaxBatch) return bad("max_batch must be 1..16");
    if (c.max_context < 1) return bad("max_context must be positive");
    if (c.n_workgroups < 1 || c.n_workgroups > 4096) return bad("n_workgroups must be 1..4096");
    if (!(c.rms_eps > 0.f) || !(c.rope_theta > 0.f)) return bad("rms_eps and rope_theta must be positive");
    d.L = c.n_layers; d.H = c.hidden; d.nq = c.n_q_heads; d.nkv = c.n_kv_heads; d.d = c.head_dim;
    d.I = c.intermediate; d.V = c.vocab; d.Bm = c.max_batch; d.Tm = c.max_context; d.G = d.nq / d.nkv;
    d.qd = d.nq * d.d; d.kvd = d.nkv * d.d; d.nqkv = d.qd + 2 * d.kvd;
    if (c.weight_bits != 0 && c.weight_bits != 16 && c.weight_bits != 4) return bad("weight_bits must be 16 or 4");
    d.w4 = c.weight_bits == 4; d.group = 0;
    if (d.w4) {
        d.group = c.group_size ? c.group_size : 128;
        if (d.group != 32 && d.group != 64 && d.group != 128) return bad("group_size must be 32, 64 or 128");
        if (d.H % d.group || d.qd % d.group || d.I % d.group) return bad("group_size must divide hidden, n_q_heads*head_dim and intermediate");
        if (d.Bm > 8) return bad("W4 weights need max_batch <= 8 in this version");
        if (d.Bm > 1 && c.use_mfma == 0) return bad("W4 weights at max_batch > 1 run on the matrix-core path only");
        if (c.ring_kb > 0) return bad("W4 weights cannot be combined with the page ring in this version");
    }
    return MK_OK;
}

static MatGeom mat_geom(int rlog, int n_rows, int k_len, int w4 = 0)
{
    MatGeom g;
    g.rlog = rlog; g.R = 1 << rlog; g.ck = (w4 ? 2048 : 512) >> rlog; g.w4 = w4;
    g.groups = ceil_div(n_rows, g.R); g.kbt = ceil_div(k_len, g.ck);
    g.n_rows = n_rows; g.k_len = k_len;
    g.S = 1; g.sm = 0;
    return g;
}

static void derive_geom(const Dims &d, const Tiling &t, Geom &g)
{
    g.qkv = mat_geom(t.r_qkv, d.nqkv, d.H, d.w4);
    g.o = mat_geom(t.r_o, d.H, d.qd, d.w4);
    const int half = (1 << t.r_gu) / 2;
    g.ipad = ceil_div(d.I, std::max(half, 4)) * std::max(half, 4);
    g.gu = mat_geom(t.r_gu, 2 * g.ipad, d.H, d.w4);
    g.down = mat_geom(t.r_d, d.H, d.I, d.w4);
    g.head = mat_geom(t.r_head, d.V, d.H);
    g.qkv.S = t.s_qkv; g.o.S = t.s_o; g.gu.S = t.s_gu; g.down.S = t.s_d;
    // O and down stage only the K range of their units: numbered slice first, the units a workgroup gets share one
    // slice (QKV and gate/up normalise the whole residual whatever their K range, so they gain nothing from it)
    g.o.sm = t.s_o > 1; g.down.sm = t.s_d > 1;
}

// ---------------------------------------------------------------- memory maps
static void plan_weights(const mk_config &c, const Dims &d, const Geom &g, WeightMap &w)
{
    uint64_t ch = 0, ve = 0;
    auto take = [&](const MatGeom &m) { uint64_t at = ch; ch += (uint64_t)m.groups * m.kbt; return (uint32_t)at; };
    auto takev = [&](uint64_t n) { uint64_t at = ve; ve += (n + 7) / 8 * 8; return (uint32_t)at; };
    w.qkv.resize(d.L); w.o.resize(d.L); w.gu.resize(d.L); w.down.resize(d.L);
    w.g_attn.resize(d.L); w.g_mlp.resize(d.L); w.bias.assign(d.L, kNone); w.qn.assign(d.L, kNone); w.kn.assign(d.L, kNone);
    for (int l = 0; l < d.L; ++l) {
        w.qkv[l] = take(g.qkv);
        w.o[l] = take(g.o);
        w.gu[l] = take(g.gu);
        w.down[l] = take(g.down);
        w.g_attn[l] = takev(d.H); w.g_mlp[l] = takev(d.H);
        if (c.qkv_bias) w.bias[l] = takev(d.nqkv);
        if (c.qk_norm) { w.qn[l] = takev(d.d); w.kn[l] = takev(d.d); }
    }
    w.n_layer_chunks = ch;
    w.embed = take(g.head);
    w.head = c.tie_embeddings ? w.embed : take(g.head);
    w.g_final = takev(d.H);
    w.n_chunks = ch; w.n_vec = ve;
}

static void plan_act(const Dims &d, const Geom &g, const Tiling &t, ActMap &a)
{
    uint64_t f = 0;
    auto take = [&](uint64_t n) { uint64_t at = f; f += (n + 63) / 64 * 64; return (uint32_t)at; };
    a.xa = take((uint64_t)d.Bm * d.H);
    a.xb = take((uint64_t)d.Bm * d.H);
    a.pqkv = take((uint64_t)t.s_qkv * d.Bm * d.nqkv);
    a.attp = take((uint64_t)d.Bm * d.nq * t.nc * (d.d + kPartPad));
    a.o = take((uint64_t)d.Bm * d.qd);
    a.po = take((uint64_t)t.s_o * d.Bm * d.H);
    a.gu = take((uint64_t)t.s_gu * d.Bm * 2 * g.ipad);
    a.pd = take((uint64_t)t.s_d * d.Bm * d.H);
    a.amax = take((uint64_t)g.head.groups * d.Bm * 2);   // at most one LM-head task per row group
    a.n_floats = f;
}

static uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

// ---------------------------------------------------------------- LDS budget (Eq. 1-2)
struct LdsBudget {
    int cap_outs;         // outputs (rows x sequences) per GEMV task the cross-wave reduction area can hold
    uint32_t red_bytes;
    uint32_t xs_cap;      // bytes left for the staged input vector
};

// Attention tasks split over the query heads of a group as well as over positions when that still
// leaves at most one task per workgroup: the score / value arithmetic of a task is proportional to
// its heads, the K/V rows are read once more (they are small next to the weights).
static int att_head_splits(const Dims &d, const Tiling &t, int n_wg)
{
    // (a matrix-core attention task scores up to 8 heads for the price of one: splitting would only re-read K and V)
    if (d.G < 2 || t.att_mc) return 1;
    const int64_t base = (int64_t)d.Bm * d.nkv * t.nc;   // tasks without a head split
    return (int)std::max<int64_t>(1, std::min<int64_t>(d.G, n_wg / base));
}

static uint32_t att_scratch_bytes(const Dims &d, const Tiling &t)
{
    if (t.att_mc)   // q, new k/v, a transposed V block (d rows of 40 bytes) per wavefront, per-wavefront merge rows (d + 4), merge weights
        return (uint32_t)((kMaxGroup + 2) * d.d + kWaves * d.G * (d.d + 4) + kWaves * kMaxGroup + 2 * kMaxGroup) * 4u + (uint32_t)(kWaves * d.d * 40);
    return (uint32_t)((kMaxGroup + 2) * d.d + kWaves * (512 / d.d) * d.G * (d.d + 4 + 1) + 2 * kMaxGroup) * 4u;   // q, new k/v, per-slot merge rows (d + 4), merge weights
}

static uint32_t norm_stage_bytes(const Dims &d, const Tiling &t)
{
    int nterm = kActTerms;
    if (t.mfma) return (uint32_t)(d.Bm * nterm) * ((uint32_t)d.H * 2u + 16u + (d.w4 ? (uint32_t)d.H / 32u * 4u : 0u));
    return (uint32_t)d.H * 4u + (d.w4 ? (uint32_t)d.H / 32u * 4u + 16u : 0u);
}

// Eq. 1: what is left of the 160 KB after the per-stage fixed areas (instruction buffer,
// semaphores/flags, reduction scratch) is available as pages; Eq. 2: the pages not pinned by the
// staged activations give the depth of the weight ring.  With ring_pages == 0 weights stream
// straight into registers and the whole remainder is available to activations.
static bool lds_budget(const Dims &d, const Tiling &t, LdsBudget &b)
{
    // reduction area: one slot per wave (matrix-core path) or per (wave, 16-lane row) (VALU path)
    b.cap_outs = t.mfma ? 1024 : 640;   // VALU: a workgroup's whole share of the LM head (about 600 rows at 256 workgroups) is one task
    // matrix-core path: room for 1536 outputs where the staged activations leave it (at batch 8 a workgroup's nine or ten
    // gate/up row groups of the 7B shape are then one task instead of two)
    if (t.mfma && kLdsMax - kLdsRed - (int64_t)kWaves * 1536 * 4 - (int64_t)t.ring_pages * t.page_bytes >=
                      std::max<int64_t>(att_scratch_bytes(d, t), norm_stage_bytes(d, t)))
        b.cap_outs = 1536;
    b.red_bytes = (uint32_t)(kWaves * (t.mfma ? 1 : 4) * b.cap_outs * 4);
    const int64_t fixed = kLdsRed + b.red_bytes;
    // pages are the 1 KB chunk slots of the ring; a pipeline stage is 16 of them
    const int64_t pages_total = pages_available(kLdsMax, 1, kLdsMisc - kLdsInstr, kLdsRed - kLdsMisc, b.red_bytes, t.page_bytes);
    const int64_t need = std::max<int64_t>(att_scratch_bytes(d, t), norm_stage_bytes(d, t));
    const int64_t pages_act = (need + t.page_bytes - 1) / t.page_bytes;
    if (t.ring_pages > 0 && pipeline_stages(pages_total, 0, 0, pages_act, 16) * 16 < t.ring_pages) return false;
    const int64_t left = kLdsMax - fixed - (int64_t)t.ring_pages * t.page_bytes;
    if (left < need) return false;
    b.xs_cap = (uint32_t)left;
    return true;
}

// ---------------------------------------------------------------- emission
struct Builder {
    const mk_config &cfg;
    const Dims &d;
    const Tiling &t;
    const Geom &g;
    const WeightMap &wm;
    const ActMap &am;
    LdsBudget lb;
    int n_wg;
    std::vector<std::vector<Instr>> lists;
    std::vector<double> load;           // accumulated chunk-equivalents per workgroup
    std::vector<uint32_t> ctr_signals;  // signals per step of every counter
    uint32_t max_xs_bytes = 0;
    int n_tasks = 0;
    uint32_t n_amax_slots = 0;          // LM-head tasks emitted so far (each owns one arg-max partial slot)

    Builder(const mk_config &c, const Dims &dd, const Tiling &tt, const Geom &gg, const WeightMap &w, const ActMap &a)
        : cfg(c), d(dd), t(tt), g(gg), wm(w), am(a), n_wg(c.n_workgroups), lists(c.n_workgroups), load(c.n_workgroups, 0.0) {}

    uint32_t new_counter() { ctr_signals.push_back(0); return (uint32_t)ctr_signals.size() - 1; }

    // workgroups ordered by accumulated load (stable), so the larger shares go to the idlest
    std::vector<int> by_load() const
    {
        std::vector<int> o(n_wg);
        std::iota(o.begin(), o.end(), 0);
        std::stable_sort(o.begin(), o.end(), [&](int a, int b) { return load[a] < load[b]; });
        return o;
    }

    uint32_t stage_bytes(uint32_t k_elems) const
    {
        int nterm = kActTerms;
        if (t.mfma) return (uint32_t)(d.Bm * nterm) * (k_elems * 2u + 16u + (d.w4 ? k_elems / 32u * 4u : 0u));   // W4: plane sums
        return k_elems * 4u + (d.w4 ? k_elems / 32u * 4u + 16u : 0u);   // W4: sums of every 32 staged values follow the vector
    }

    // LDS bytes a PRO_COMBINE task needs behind its staged vector of k_elems values: the partial rows
    // [head][chunk][d + pad] of the heads covering the k range (one sequence at a time) and their weights.
    uint32_t combine_bytes(uint32_t k_elems) const
    {
        const uint32_t nh = (k_elems + (uint32_t)d.d - 1) / (uint32_t)d.d;
        return nh * (uint32_t)t.nc * (uint32_t)(d.d + kPartPad + 1) * 4u + 16u;
    }

    // Partition the units of one GEMV operator instance over the workgroups and emit its tasks.
    // `proto` carries everything except u0/nu/staged range/skip flag/signal.  Returns false if a task cannot fit LDS.
    bool emit_gemv(Instr proto, const MatGeom &m, uint32_t wait_ctr, uint32_t sig_ctr)
    {
        const uint32_t S = proto.S, kbt = proto.kbt, nkb = proto.nkb;
        const uint32_t U = (uint32_t)m.groups * S;
        const int parts = (int)std::min<uint32_t>((uint32_t)n_wg, U);
        const uint32_t pro = instr_pro(proto);
        const bool normk = pro == PRO_EMBED_NORM || pro == PRO_RESID_NORM;
        const bool store_slice = normk && proto.xs_out != kNone;
        const int cols = t.mfma ? d.Bm : 1;
        const uint32_t cap_units = std::max<uint32_t>(1, (uint32_t)lb.cap_outs / (uint32_t)(m.R * cols));
        std::vector<int> order = by_load();
        uint32_t base = U / parts, rem = U % parts, u = 0;
        for (int pi = 0; pi < parts; ++pi) {
            const int wg = order[pi];
            uint32_t share = base + ((uint32_t)pi < rem ? 1u : 0u);
            uint32_t u_end = u + share;
            bool first = true;
            uint32_t prev_lo = kNone, prev_n = kNone;
            while (u < u_end) {
                // grow the task unit by unit while the reduction area and the staged input fit
                uint32_t nu = 0, klo = 0, khi = 0;
                while (u + nu < u_end && nu < cap_units) {
                    uint32_t uu = u + nu, rg, s;
                    unit_place(m.sm != 0, uu, S, (uint32_t)m.groups, rg, s);
                    uint32_t lo = s * nkb, hi = (s == S - 1) ? kbt : lo + nkb;
                    uint32_t nlo = nu ? std::min(klo, lo) : lo, nhi = nu ? std::max(khi, hi) : hi;
                    if (!normk && stage_bytes((nhi - nlo) * m.ck) + (pro == PRO_COMBINE ? combine_bytes((nhi - nlo) * m.ck) : 0u) > lb.xs_cap) break;
                    klo = nlo; khi = nhi; ++nu;
                }
                if (nu == 0) return false;
                Instr I = proto;
                I.u0 = u; I.nu = nu;
                I.wait_ctr[0] = wait_ctr; I.wait_ctr[1] = kNone;
                I.wait_cnt[0] = wait_ctr == kNone ? 0 : ctr_signals[wait_ctr];
                if (I.flags & F_WAIT_PREV) I.wait_cnt[0] = (uint32_t)d.Bm;   // the arg-max counter: one signal per sequence
                I.wait_cnt[1] = 0;
                if (I.flags & F_ARGMAX) I.spare = n_amax_slots++;
                I.sig_ctr = kNone;
                if (normk) {
                    // the first task of each participant stores its 4-aligned slice of the new residual
                    I.xs_lo = I.xs_hi = 0;
                    if (first && store_slice) {
                        I.xs_lo = 4u * (uint32_t)((uint64_t)(d.H / 4) * pi / parts);
                        I.xs_hi = 4u * (uint32_t)((uint64_t)(d.H / 4) * (pi + 1) / parts);
                    }
                    if (!store_slice) I.xs_out = 0;
                    if (!first) I.flags |= F_SKIP_PRO;
                    max_xs_bytes = std::max(max_xs_bytes, norm_stage_bytes(d, t));
                } else {
                    I.xs_lo = klo; I.xs_hi = khi - klo;
                    if (!first && prev_lo == I.xs_lo && prev_n == I.xs_hi) I.flags |= F_SKIP_PRO;
                    prev_lo = I.xs_lo; prev_n = I.xs_hi;
                    uint32_t need = stage_bytes((khi - klo) * m.ck);
                    if (pro == PRO_COMBINE) {
                        I.in_base = (need + 15u) & ~15u;                    // partial rows are staged behind the vector
                        need = I.in_base + combine_bytes((khi - klo) * m.ck);
                    }
                    max_xs_bytes = std::max(max_xs_bytes, need);
                }
                if (u + nu == u_end) { I.sig_ctr = sig_ctr; if (sig_ctr != kNone) ++ctr_signals[sig_ctr]; }
                lists[wg].push_back(I);
                ++n_tasks;
                // load: chunks streamed + a fixed per-task cost (in chunk equivalents)
                const uint32_t c0 = unit_chunk0(m.sm != 0, u, S, (uint32_t)m.groups, kbt, nkb);
                const uint32_t c1 = unit_chunk0(m.sm != 0, u + nu, S, (uint32_t)m.groups, kbt, nkb);
                load[wg] += (double)(c1 - c0) + 4.0;
                u += nu; first = false;
            }
        }
        return true;
    }

    Instr gemv_proto(uint32_t stage, int l, const MatGeom &m, uint32_t w_chunk, int S, uint32_t pro, uint32_t n_parts,
                     uint32_t prod_rlog) const
    {
        Instr I{};
        I.op = OP_GEMV; I.flags = (t.mfma ? F_MFMA : 0u) | (m.w4 ? F_W4 : 0u) | (m.sm ? F_SLICE_MAJOR : 0u); I.ref_seq = (uint32_t)l * 8 + stage; I.layer = (uint32_t)l;
        I.w_chunk = w_chunk; I.kbt = (uint32_t)m.kbt; I.S = (uint32_t)S; I.nkb = (uint32_t)ceil_div(m.kbt, S);
        I.n_rows = (uint32_t)m.n_rows; I.k_len = (uint32_t)m.k_len;
        I.cfg = make_cfg(pro, (uint32_t)m.rlog, prod_rlog, n_parts);
        I.bias = kNone; I.xs_out = kNone;
        return I;
    }

    bool build()
    {
        if (!lds_budget(d, t, lb)) return false;
        // The residual stream lives in xa / xb.  `res` is the buffer holding the current residual,
        // `parts` the K-split partial sums still to be added to it (summed in the next prologue).
        uint32_t res = am.xa, parts_off = 0, parts_n = 0;
        // Counter of the greedy-token tasks that close a step.  The first tasks of the NEXT step wait
        // for it (F_WAIT_PREV), which orders whole steps inside a multi-step launch.
        const uint32_t c_argmax = new_counter();
        uint32_t prev_done = c_argmax;
        auto other = [&](uint32_t b) { return b == am.xa ? am.xb : am.xa; };
        for (int l = 0; l < d.L; ++l) {
            const uint32_t c_qkv = new_counter(), c_comb = new_counter(), c_o = new_counter(), c_gu = new_counter(),
                           c_d = new_counter();
            // attention tasks signal one counter per (sequence, kv head) for the combine tasks, or, when the
            // O projection combines the partials itself, one counter per layer
            std::vector<uint32_t> c_att(d.Bm * d.nkv);
            const uint32_t c_att_layer = t.fuse ? new_counter() : kNone;
            for (auto &c : c_att) c = t.fuse ? c_att_layer : new_counter();

            // ---- QKV projection: prologue = (embedding | residual + pending partials) -> RMSNorm
            {
                Instr q = gemv_proto(ST_QKV, l, g.qkv, wm.qkv[l], t.s_qkv, l == 0 ? PRO_EMBED_NORM : PRO_RESID_NORM, parts_n, 0);
                q.in_base = res; q.in_parts = parts_off; q.part_stride = d.Bm * d.H; q.in_ld = d.H;
                if (l == 0) { q.xs_out = am.xa; res = am.xa; }
                else if (parts_n) { q.xs_out = other(res); res = other(res); }
                parts_n = 0;
                q.gain = wm.g_attn[l];
                q.out = am.pqkv; q.out_split_stride = d.Bm * d.nqkv; q.out_ld = d.nqkv; q.bias = wm.bias[l];
                if (l == 0) q.flags |= F_WAIT_PREV;
                if (!emit_gemv(q, g.qkv, prev_done, c_qkv)) return false;
            }
            // ---- attention partials: one task per (sequence, kv head, chunk)
            {
                std::vector<int> order = by_load();
                int oi = 0;
                const int hs = att_head_splits(d, t, n_wg);
                for (int b = 0; b < d.Bm; ++b)
                    for (int gh = 0; gh < d.nkv; ++gh)
                        for (int c = 0; c < t.nc; ++c)
                        for (int hp = 0; hp < hs; ++hp) {
                            InstrAtt a{};
                            // heads [h0, h0 + nh) of the group: G / hs each, the first G % hs parts one more
                            const int h_base = d.G / hs, h_rem = d.G % hs;
                            const int h_lo = hp * h_base + std::min(hp, h_rem), h_n = h_base + (hp < h_rem ? 1 : 0);
                            a.h0 = (uint32_t)h_lo; a.nh = (uint32_t)h_n;
                            a.op = OP_ATT; a.ref_seq = l * 8 + ST_ATT; a.layer = l; a.flags = t.att_mc ? F_ATT_MC : 0u;
                            a.wait_ctr[0] = c_qkv; a.wait_cnt[0] = ctr_signals[c_qkv]; a.wait_ctr[1] = kNone;
                            a.sig_ctr = c_att[b * d.nkv + gh]; ++ctr_signals[a.sig_ctr];
                            a.b = b; a.g = gh; a.c = c; a.nc = t.nc; a.bs = t.bs;
                            a.in_parts = am.pqkv; a.n_parts = t.s_qkv; a.part_stride = d.Bm * d.nqkv; a.in_ld = d.nqkv;
                            a.qn_gain = wm.qn[l]; a.kn_gain = wm.kn[l];
                            a.out = am.attp;
                            int wg = order[oi % n_wg]; ++oi;
                            Instr raw; memcpy(&raw, &a, sizeof raw);
                            lists[wg].push_back(raw); ++n_tasks;
                            load[wg] += (double)d.Tm / t.nc * d.d * 4.0 / kChunkBytes * 0.5 + 8.0;
                        }
            }
            // ---- combine: one task per (sequence, q head)
            if (!t.fuse) {
                std::vector<int> order = by_load();
                int oi = 0;
                for (int b = 0; b < d.Bm; ++b)
                    for (int h = 0; h < d.nq; ++h) {
                        InstrAtt a{};
                        a.op = OP_COMB; a.ref_seq = l * 8 + ST_COMB; a.layer = l;
                        uint32_t ca = c_att[b * d.nkv + h / d.G];
                        a.wait_ctr[0] = ca; a.wait_cnt[0] = ctr_signals[ca]; a.wait_ctr[1] = kNone;
                        a.sig_ctr = c_comb; ++ctr_signals[c_comb];
                        a.b = b; a.nc = t.nc; a.out = am.attp; a.h0 = h; a.nh = 1; a.o_out = am.o; a.o_ld = d.qd;
                        int wg = order[oi % n_wg]; ++oi;
                        Instr raw; memcpy(&raw, &a, sizeof raw);
                        lists[wg].push_back(raw); ++n_tasks;
                        load[wg] += 4.0;
                    }
            }
            // ---- O projection; unsplit: the epilogue adds the residual, split: partials for the next prologue
            {
                Instr o = gemv_proto(ST_O, l, g.o, wm.o[l], t.s_o, t.fuse ? PRO_COMBINE : PRO_PLAIN, t.fuse ? t.nc : 1, 0);
                o.in_parts = t.fuse ? am.attp : am.o; o.part_stride = 0; o.in_ld = d.qd;
                o.out_ld = d.H;
                if (t.s_o == 1) { o.flags |= F_ADD_RESID; o.resid = res; o.out = other(res); res = other(res); }
                else { o.out = am.po; o.out_split_stride = d.Bm * d.H; parts_off = am.po; parts_n = t.s_o; }
                if (!emit_gemv(o, g.o, t.fuse ? c_att_layer : c_comb, c_o)) return false;
            }
            // ---- gate/up projection: prologue = residual (+ O partials) -> RMSNorm; unsplit: SiLU * up in the epilogue
            {
                Instr gu = gemv_proto(ST_GU, l, g.gu, wm.gu[l], t.s_gu, PRO_RESID_NORM, parts_n, 0);
                gu.in_base = res; gu.in_parts = parts_off; gu.part_stride = d.Bm * d.H; gu.in_ld = d.H;
                if (parts_n) { gu.xs_out = other(res); res = other(res); }
                parts_n = 0;
                gu.gain = wm.g_mlp[l];
                gu.out = am.gu;
                if (t.s_gu == 1) { gu.flags |= F_SILU_EPI; gu.out_ld = g.ipad; }
                else { gu.out_split_stride = d.Bm * 2 * g.ipad; gu.out_ld = 2 * g.ipad; }
                if (!emit_gemv(gu, g.gu, c_o, c_gu)) return false;
            }
            // ---- down projection
            {
                const bool fused = t.s_gu == 1;
                Instr dn = gemv_proto(ST_DOWN, l, g.down, wm.down[l], t.s_d, fused ? PRO_PLAIN : PRO_SILU,
                                      fused ? 1 : t.s_gu, (uint32_t)g.gu.rlog);
                dn.in_parts = am.gu; dn.part_stride = fused ? 0 : d.Bm * 2 * g.ipad; dn.in_ld = fused ? g.ipad : 2 * g.ipad;
                dn.out_ld = d.H;
                if (t.s_d == 1) { dn.flags |= F_ADD_RESID; dn.resid = res; dn.out = other(res); res = other(res); }
                else { dn.out = am.pd; dn.out_split_stride = d.Bm * d.H; parts_off = am.pd; parts_n = t.s_d; }
                if (!emit_gemv(dn, g.down, c_gu, c_d)) return false;
            }
            prev_done = c_d;
            // ---- residual sum: one level in which each workgroup adds its slice of the down projection's partial rows to
            //      the residual, instead of every task of the next operator reading all of them
            if (parts_n && wants_residual_sum(t.s_d, d.Bm, d.H)) {
                const uint32_t c_rs = new_counter();
                const int np = std::min(n_wg, d.H / 4);
                std::vector<int> order = by_load();
                for (int pi = 0; pi < np; ++pi) {
                    Instr r{};
                    r.op = OP_RSUM; r.ref_seq = (uint32_t)l * 8 + ST_RSUM; r.layer = (uint32_t)l;
                    r.wait_ctr[0] = c_d; r.wait_cnt[0] = ctr_signals[c_d]; r.wait_ctr[1] = kNone;
                    r.sig_ctr = c_rs; ++ctr_signals[c_rs];
                    r.cfg = make_cfg(0, 0, 0, parts_n);
                    r.in_base = res; r.in_parts = parts_off; r.part_stride = (uint32_t)(d.Bm * d.H); r.in_ld = (uint32_t)d.H;
                    r.xs_lo = 4u * (uint32_t)((uint64_t)(d.H / 4) * pi / np);
                    r.xs_hi = 4u * (uint32_t)((uint64_t)(d.H / 4) * (pi + 1) / np);
                    r.xs_out = other(res);
                    lists[order[pi]].push_back(r); ++n_tasks;
                    load[order[pi]] += 2.0;
                }
                res = other(res); parts_n = 0; prev_done = c_rs;
            }
        }
        // ---- final norm + LM head (never stores a residual slice)
        Instr h = gemv_proto(ST_HEAD, d.L, g.head, wm.head, 1, PRO_RESID_NORM, parts_n, 0);
        h.flags |= F_LOGITS | F_ARGMAX;
        h.in_base = res; h.in_parts = parts_off; h.part_stride = d.Bm * d.H; h.in_ld = d.H;
        h.gain = wm.g_final; h.out_ld = d.V;
        const uint32_t c_head = new_counter();
        if (!emit_gemv(h, g.head, prev_done, c_head)) return false;
        // ---- greedy token: one task per sequence reduces the (max, row) partials of the LM-head tasks
        {
            std::vector<int> order = by_load();
            for (int b = 0; b < d.Bm; ++b) {
                InstrAtt a{};
                a.op = OP_ARGMAX; a.ref_seq = d.L * 8 + ST_ARGMAX; a.layer = d.L;
                a.wait_ctr[0] = c_head; a.wait_cnt[0] = ctr_signals[c_head]; a.wait_ctr[1] = kNone;
                a.sig_ctr = c_argmax; ++ctr_signals[c_argmax];
                a.b = b; a.out = am.amax; a.n_slots = n_amax_slots;
                Instr raw; memcpy(&raw, &a, sizeof raw);
                lists[order[b % n_wg]].push_back(raw); ++n_tasks;
                load[order[b % n_wg]] += 2.0;
            }
        }
        max_xs_bytes = std::max(max_xs_bytes, att_scratch_bytes(d, t));
        max_xs_bytes = std::max(max_xs_bytes, (uint32_t)(t.nc * (d.d + kPartPad + 1) * 4));   // combine task: partial rows + merge weights
        return true;
    }
};

// A split must leave every unit at least one chunk; ragged last units are fine.
static bool split_ok(int kbt, int s) { return s >= 1 && s <= kbt && ceil_div(kbt, s) * (s - 1) < kbt; }

// ---------------------------------------------------------------- replay (shared by simulator and verifier)
// Walks the per-workgroup lists as the kernel does: a task may start when all the counters it
// waits on have received their signals.  visit(wg, idx, instr) is called in a valid execution
// order.  Returns false on deadlock (some list cannot finish).
template <class F>
static bool replay(const mk_schedule *s, F &&visit, std::string *why)
{
    const int n_wg = s->n_wg, mi = s->max_instr;
    std::vector<int> pc(n_wg, 0);
    std::vector<uint32_t> got(s->n_counters, 0);
    const Instr *all = (const Instr *)s->instr.data();
    bool progress = true;
    size_t remaining = 0;
    for (int w = 0; w < n_wg; ++w)
        for (int i = 0; i < mi && all[(size_t)w * mi + i].op != OP_END; ++i) ++remaining;
    while (remaining && progress) {
        progress = false;
        for (int w = 0; w < n_wg; ++w) {
            while (pc[w] < mi) {
                const Instr &I = all[(size_t)w * mi + pc[w]];
                if (I.op == OP_END) break;
                bool ready = true;
                for (int k = 0; k < 2; ++k)
                    if (I.wait_ctr[k] != kNone) {
                        if (I.wait_ctr[k] >= (uint32_t)s->n_counters) { if (why) *why = "wait on a counter that does not exist"; return false; }
                        if (k == 0 && (I.flags & F_WAIT_PREV)) continue;   // satisfied by the previous step
                        if (got[I.wait_ctr[k]] < I.wait_cnt[k]) ready = false;
                    }
                if (!ready) break;
                visit(w, pc[w], I);
                if (I.sig_ctr != kNone) {
                    if (I.sig_ctr >= (uint32_t)s->n_counters) { if (why) *why = "signal to a counter that does not exist"; return false; }
                    ++got[I.sig_ctr];
                }
                ++pc[w]; --remaining; progress = true;
            }
        }
    }
    if (remaining) {
        if (why) {
            char buf[160];
            for (int w = 0; w < n_wg; ++w) {
                const Instr &I = all[(size_t)w * mi + pc[w]];
                if (pc[w] < mi && I.op != OP_END) {
                    snprintf(buf, sizeof buf, "deadlock: workgroup %d stuck at instruction %d (ref_seq %u) waiting on counter %u",
                             w, pc[w], I.ref_seq, I.wait_ctr[0]);
                    *why = buf;
                    break;
                }
            }
        }
        return false;
    }
    return true;
}

static uint32_t task_chunks(const Instr &I)
{
    const bool sm = (I.flags & F_SLICE_MAJOR) != 0;
    const uint32_t groups = instr_groups(I);
    return unit_chunk0(sm, I.u0 + I.nu, I.S, groups, I.kbt, I.nkb) - unit_chunk0(sm, I.u0, I.S, groups, I.kbt, I.nkb);
}

// Pipeline cost model (Sec. 4.2.2 Step 3-4).  Per workgroup two timelines: the weight stream
// (HBM -> registers / LDS pages) and the consumer.  Without an LDS ring only the first
// prefetch window of a task overlaps its dependency wait; with a ring the stream runs ahead of
// the consumer by up to the ring capacity (page states: Locked while loading, Ready once
// landed, Empty again when consumed).
static SimResult simulate(const mk_schedule *s)
{
    const double bw_chip = 8.0e6 * 0.70;                         // bytes per microsecond the chip sustains
    const double bw_wg = bw_chip / s->n_wg;
    const double sync_us = 1.8, pro_us_per_kfloat = 0.02, task_us = 0.6, sig_us = 0.8;
    const double ring_bytes = (double)s->tl.ring_pages * s->tl.page_bytes;
    const double window = ring_bytes > 0 ? ring_bytes : (double)(kPrefetch * kWaves * kChunkBytes);
    std::vector<double> t_cons(s->n_wg, 0.0), t_load(s->n_wg, 0.0), busy(s->n_wg, 0.0);
    std::vector<double> ctr_done(s->n_counters, 0.0);
    const Dims &d = s->dm;
    replay(s, [&](int w, int, const Instr &I) {
        double dep = 0.0;
        for (int k = 0; k < 2; ++k)
            if (I.wait_ctr[k] != kNone && !(k == 0 && (I.flags & F_WAIT_PREV))) dep = std::max(dep, ctr_done[I.wait_ctr[k]] + sync_us);
        double bytes = 0.0, pro = 0.0;
        if (I.op == OP_GEMV) {
            bytes = (double)task_chunks(I) * kChunkBytes;
            if (!(I.flags & F_SKIP_PRO)) {
                const uint32_t pr = instr_pro(I), np = instr_nparts(I);
                const bool normk = pr == PRO_EMBED_NORM || pr == PRO_RESID_NORM;
                double fl = normk ? (double)d.H * (1 + np) : (double)I.xs_hi * instr_ck(I) * np * (pr == PRO_SILU ? 2 : 1);
                // one memory round trip per four partials in flight, plus the bytes themselves
                pro = 0.8 + 0.8 * ((np + 3) / 4) + fl * d.Bm / 1000.0 * pro_us_per_kfloat;
                if (pr == PRO_COMBINE) pro = 1.6 + fl * d.Bm / 1000.0 * pro_us_per_kfloat;   // all partial rows in flight at once
                if (s->tl.mfma && pr != PRO_COMBINE) {
                    // matrix-core staging, fitted to task traces at batch 4 and 8 (1.5B and 7B shapes): every float read
                    // past the caches costs about 0.07 us per thousand, every staged value (split into two bf16 planes)
                    // 0.1 us per thousand, the normalising forms one more pass over LDS
                    const double loaded = fl * d.Bm / 1000.0;
                    const double staged = (normk ? (double)d.H : (double)I.xs_hi * instr_ck(I)) * d.Bm / 1000.0;
                    pro = 0.9 + 0.07 * loaded + 0.1 * staged + (normk ? 0.8 : 0.0);
                }
            }
            // units are flushed through a cross-lane reduction: small R means more flushes per byte
            pro += 0.004 * I.nu;
        } else if (I.op == OP_ATT) {
            bytes = (double)d.Tm / s->tl.nc * d.d * 4.0;
            pro = s->tl.att_mc ? 2.4 : 0.5;   // (matrix-core form: q staging as bf16 columns and the per-wavefront merge)
        } else if (I.op == OP_COMB) {
            pro = 0.3 + s->tl.nc * 0.01;
        } else if (I.op == OP_RSUM) {
            pro = 1.2;   // one round trip for the base and partial rows of a slice
        } else {
            pro = 1.0;   // arg-max over the LM-head partials
        }
        // weight stream: may start once the ring has room, i.e. `window` bytes ahead of the consumer
        double lead = std::min(bytes, window);
        double load_start = std::max(t_load[w], t_cons[w] - lead / bw_wg);   // earliest the stream can begin this task
        load_start = std::max(load_start, 0.0);
        double start = std::max(t_cons[w], dep);
        // bytes beyond the window can only stream while the consumer drains
        double stream_end = std::max(load_start + lead / bw_wg, start + pro) + (bytes - lead) / bw_wg;
        double end = std::max(start + pro, stream_end) + task_us + (I.sig_ctr != kNone ? sig_us : 0.0);
        busy[w] += bytes / bw_wg;
        t_load[w] = stream_end;
        t_cons[w] = end;
        if (I.sig_ctr != kNone) ctr_done[I.sig_ctr] = std::max(ctr_done[I.sig_ctr], end);
    }, nullptr);
    SimResult r;
    r.makespan_us = *std::max_element(t_cons.begin(), t_cons.end());
    double b = std::accumulate(busy.begin(), busy.end(), 0.0);
    r.duty = r.makespan_us > 0 ? b / (r.makespan_us * s->n_wg) : 0.0;
    return r;
}

// ---------------------------------------------------------------- assemble a schedule object from a tiling
static int assemble(const mk_config &cfg, const Dims &d, const Tiling &t, mk_schedule *s)
{
    s->cfg = cfg; s->dm = d; s->tl = t;
    derive_geom(d, t, s->gm);
    plan_weights(cfg, d, s->gm, s->wm);
    plan_act(d, s->gm, t, s->am);
    Builder b(cfg, d, t, s->gm, s->wm, s->am);
    if (!b.build()) return MK_EINFEASIBLE;
    s->n_wg = cfg.n_workgroups;
    size_t mx = 0;
    for (auto &l : b.lists) mx = std::max(mx, l.size());
    s->max_instr = (int)mx + 1;
    s->n_counters = (int)b.ctr_signals.size();
    s->n_tasks = b.n_tasks;
    s->instr.assign((size_t)s->n_wg * s->max_instr * kInstrDwords, 0u);
    std::vector<uint32_t> seqs;
    for (int w = 0; w < s->n_wg; ++w) {
        memcpy(s->instr.data() + (size_t)w * s->max_instr * kInstrDwords, b.lists[w].data(), b.lists[w].size() * sizeof(Instr));
        for (auto &I : b.lists[w]) seqs.push_back(I.ref_seq);
    }
    std::sort(seqs.begin(), seqs.end());
    seqs.erase(std::unique(seqs.begin(), seqs.end()), seqs.end());
    s->ref_seqs = seqs;
    s->lds_red_bytes = b.lb.red_bytes;
    s->lds_xs_off = kLdsRed + b.lb.red_bytes;
    s->lds_ring_off = (uint32_t)align_up(s->lds_xs_off + b.max_xs_bytes, 1024);
    s->lds_ring_slots = (uint32_t)((uint64_t)t.ring_pages * t.page_bytes / kChunkBytes);
    s->lds_total = t.ring_pages ? s->lds_ring_off + s->lds_ring_slots * kChunkBytes
                                : (uint32_t)align_up(s->lds_xs_off + b.max_xs_bytes, 256);
    if (s->lds_total > (uint64_t)kLdsMax) return MK_EINFEASIBLE;
    // workspace layout
    Layout &L = s->lay;
    uint64_t off = 0;
    L.weights = off; off = align_up(off + s->wm.n_chunks * kChunkBytes, 4096);
    L.wscale = off; off = align_up(off + (d.w4 ? s->wm.n_layer_chunks * (2048u / d.group) * 2 : 0), 4096);
    L.vecs = off; off = align_up(off + s->wm.n_vec * 2, 4096);
    L.rope = off; off = align_up(off + (uint64_t)d.Tm * d.d * 4, 4096);
    L.act = off; off = align_up(off + s->am.n_floats * 4, 4096);
    L.counters = off; off = align_up(off + (uint64_t)s->n_counters * kCounterDwords * 4, 4096);
    L.instr = off; off = align_up(off + s->instr.size() * 4, 4096);
    L.err = off; off = align_up(off + 64, 4096);
    L.trace = off; off = align_up(off + ((cfg.flags & MK_F_TRACE) ? (uint64_t)s->n_wg * s->max_instr * 64 : 0), 4096);
    L.stream = off; off = align_up(off + (uint64_t)s->n_wg * s->max_instr * 8, 4096);
    L.tokens = off; off = align_up(off + (uint64_t)kMaxBatch * 4, 4096);
    L.total = off;
    s->sim = simulate(s);
    return MK_OK;
}

// ---------------------------------------------------------------- recorded profile-guided tilings
// Sec. 4.2.2 Step 4: candidates are profiled offline on the target GPU and the best trace is locked in.
// The on-device search (autotune.py, through this same C ABI) records its winner per deployment
// configuration in a text table next to the library: one line per configuration,
//     <L>-<H>-<nq>-<nkv>-<d>-<I>-<V>-<max_batch>-wg<workgroups>-w<weight bits>  name=value ...
// with the names of the tiling fields of mk_config.  mk_build_schedule applies a matching line when
// the caller fixes no tiling field itself, so that the schedule it returns is the profiled one.
std::string tuned_key(const mk_config &c)
{
    char buf[200];
    snprintf(buf, sizeof buf, "%d-%d-%d-%d-%d-%d-%d-%d-wg%d-w%d", c.n_layers, c.hidden, c.n_q_heads, c.n_kv_heads, c.head_dim,
             c.intermediate, c.vocab, c.max_batch, c.n_workgroups, c.weight_bits == 4 ? 4 : 16);
    return buf;
}

std::string tuned_table_path()
{
    if (const char *e = getenv("MK_TUNED_TABLE")) return e;      // read when a schedule is built, never on the launch path
    Dl_info info;
    if (!dladdr((const void *)&tuned_table_path, &info) || !info.dli_fname) return "";
    std::string p = info.dli_fname;
    const size_t slash = p.rfind('/');
    return (slash == std::string::npos ? std::string(".") : p.substr(0, slash)) + "/tuned_tilings.txt";
}

static bool names_no_tiling(const mk_config &c)
{
    return !c.split_qkv && !c.split_o && !c.split_gateup && !c.split_down && !c.attn_chunks && !c.chunk_rows && !c.rows_qkv &&
           !c.rows_o && !c.rows_gateup && !c.rows_down && !c.rows_head && c.fuse_combine <= 0 && c.ring_kb <= 0 && c.use_mfma < 0;
}

// Applies the recorded line of this configuration to `c`; false when there is none (or the table is absent).
static bool apply_tuned(mk_config &c)
{
    const std::string path = tuned_table_path();
    if (path.empty()) return false;
    std::ifstream f(path);
    if (!f) return false;
    const std::string key = tuned_key(c);
    std::string line;
    while (std::getline(f, line)) {
        const size_t hash = line.find('#');
        if (hash != std::string::npos) line.resize(hash);
        std::istringstream is(line);
        std::string k, kv;
        if (!(is >> k) || k != key) continue;
        mk_config t = c;
        struct { const char *name; int32_t mk_config::*field; } names[] = {
            {"split_qkv", &mk_config::split_qkv}, {"split_o", &mk_config::split_o}, {"split_gateup", &mk_config::split_gateup},
            {"split_down", &mk_config::split_down}, {"attn_chunks", &mk_config::attn_chunks}, {"rows_qkv", &mk_config::rows_qkv},
            {"rows_o", &mk_config::rows_o}, {"rows_gateup", &mk_config::rows_gateup}, {"rows_down", &mk_config::rows_down},
            {"rows_head", &mk_config::rows_head}, {"fuse_combine", &mk_config::fuse_combine}};
        bool ok = true;
        while (is >> kv) {
            const size_t eq = kv.find('=');
            if (eq == std::string::npos) { ok = false; break; }
            const std::string name = kv.substr(0, eq);
            if (name == "ms") continue;                             // the measured step time, informative only
            char *end = nullptr;
            const long v = strtol(kv.c_str() + eq + 1, &end, 10);
            if (!end || *end || v < 0 || v > 4096) { ok = false; break; }
            bool known = false;
            for (auto &n : names)
                if (name == n.name) { t.*(n.field) = (int32_t)v; known = true; }
            if (!known) { ok = false; break; }
        }
        if (!ok) continue;      // a malformed line is ignored: the cost model's choice stands
        c = t;
        return true;
    }
    return false;
}

int build_schedule(const mk_config *cfg_in, mk_schedule **out)
{
    if (!cfg_in || !out) { set_error("null argument"); return MK_EINVAL; }
    mk_config cfg = *cfg_in;
    Dims d;
    int rc = derive_dims(cfg, d);
    if (rc) return rc;
    // no tiling fixed by the caller: the profiled choice recorded for this configuration, if any (a
    // recorded line that no longer builds falls back to the cost model's search below)
    if (!(cfg.flags & MK_F_NO_TABLE) && names_no_tiling(cfg)) {
        mk_config t = cfg;
        if (apply_tuned(t)) {
            t.flags |= MK_F_NO_TABLE;
            mk_schedule *s = nullptr;
            if (build_schedule(&t, &s) == MK_OK) {
                s->cfg.flags = cfg.flags;
                s->from_table = 1;
                *out = s;
                return MK_OK;
            }
        }
    }
    // auto: matrix cores when several sequences make the projections a thin GEMM.  At batch 1 the VALU forms measure
    // faster for bf16 and for W4 alike (1.14 against 1.48 ms per step for W4 at the 1.5B shape): the matrix-core form
    // needs 16 rows per chunk, which leaves the small projections with 96-128 tasks for 256 workgroups, and its
    // prologue stages bf16 planes.
    const int mfma = cfg.use_mfma < 0 ? (d.Bm > 1 ? 1 : 0) : (cfg.use_mfma ? 1 : 0);
    if (!mfma && d.Bm > 1) { set_error("mk_config: the VALU GEMV path handles max_batch == 1 only"); return MK_EINVAL; }
    if (cfg.ring_kb < -2 || (cfg.ring_kb > 0 && (cfg.ring_kb < 16 || cfg.ring_kb > 144))) { set_error("mk_config: ring_kb must be -2 (search), -1 (auto), 0 (no ring) or 16..144"); return MK_EINVAL; }

    for (int v : {cfg.split_qkv, cfg.split_o, cfg.split_gateup, cfg.split_down, cfg.attn_chunks})
        if (v < 0) { set_error("mk_config: negative split / chunk count"); return MK_EINVAL; }
    auto opt = [](int fixed, std::initializer_list<int> opts) {
        return fixed > 0 ? std::vector<int>{fixed} : std::vector<int>(opts);
    };
    std::vector<int> c_sqkv = opt(cfg.split_qkv, {1, 2}), c_so = opt(cfg.split_o, {1, 2, 4}),
                     c_sgu = opt(cfg.split_gateup, {1, 2}), c_sd = opt(cfg.split_down, {1, 2, 4, 8});
    // rows per weight chunk: the matrix-core path needs 16; the VALU path may trade rows for K
    std::vector<int> c_r = mfma ? std::vector<int>{4} : std::vector<int>{4, 3, 2, 1};
    std::vector<int> c_rgu = mfma ? std::vector<int>{4} : std::vector<int>{4, 3, 2};
    auto rows_log = [](int rows) { return rows == 2 ? 1 : rows == 4 ? 2 : rows == 8 ? 3 : rows == 16 ? 4 : -1; };
    if (cfg.chunk_rows) {
        int rl = rows_log(cfg.chunk_rows);
        if (rl < 0 || (mfma && rl != 4)) { set_error("mk_config: chunk_rows must be 2, 4, 8 or 16 (16 on the matrix-core path)"); return MK_EINVAL; }
        c_r = {rl}; c_rgu = {rl};
    }
    // per-matrix overrides
    std::vector<int> c_rq = c_r, c_ro = c_r, c_rd = c_r, c_rh = {cfg.chunk_rows ? c_r[0] : 4};
    struct RowOpt { int rows; std::vector<int> *dst; int min_log; };
    for (RowOpt o : {RowOpt{cfg.rows_qkv, &c_rq, 1}, RowOpt{cfg.rows_o, &c_ro, 1}, RowOpt{cfg.rows_gateup, &c_rgu, 1},
                     RowOpt{cfg.rows_down, &c_rd, 1}, RowOpt{cfg.rows_head, &c_rh, 1}}) {
        if (!o.rows) continue;
        int rl = rows_log(o.rows);
        if (rl < o.min_log || (mfma && rl != 4)) { set_error("mk_config: rows_* must be 2, 4, 8 or 16 (16 on the matrix-core path)"); return MK_EINVAL; }
        *o.dst = {rl};
    }
    std::vector<int> c_nc;
    if (cfg.attn_chunks > 0) c_nc.push_back(cfg.attn_chunks);
    else
        for (int nc = 1; nc <= 64; nc *= 2) {   // (the combine task stages nc partial rows in LDS)
            if ((int64_t)d.Bm * d.nkv * nc > 2 * (int64_t)cfg.n_workgroups && nc > 1) break;
            c_nc.push_back(nc);
        }

    // A candidate is admissible when every K split leaves no empty unit, the norm-prologue
    // operators have K a whole number of chunks, and the split gate/up path keeps 128-bit rows.
    auto admissible = [&](const Tiling &t) {
        Geom g;
        derive_geom(d, t, g);
        if (d.H % g.qkv.ck || d.H % g.gu.ck || d.H % g.head.ck) return false;
        if (d.nqkv % g.qkv.R || d.qd % g.qkv.R || d.kvd % g.qkv.R) return false;
        if (!split_ok(g.qkv.kbt, t.s_qkv) || !split_ok(g.o.kbt, t.s_o) || !split_ok(g.gu.kbt, t.s_gu) || !split_ok(g.down.kbt, t.s_d)) return false;
        if (t.s_gu > 1 && g.gu.R < 8) return false;
        // a fused combine stages whole heads: every K split of the O projection must start and end on a head
        if (t.fuse && t.s_o > 1 && (ceil_div(g.o.kbt, t.s_o) * g.o.ck) % d.d) return false;
        if (t.fuse && t.nc > 64) return false;
        return true;
    };

    // coordinate descent over the tiling parameters, each candidate scored by the simulator
    Tiling best{};
    best.s_qkv = c_sqkv[0]; best.s_o = c_so[0]; best.s_gu = c_sgu[0]; best.s_d = c_sd[0];
    best.r_qkv = c_rq[0]; best.r_o = c_ro[0]; best.r_gu = c_rgu[0]; best.r_d = c_rd[0]; best.r_head = c_rh[0];
    best.nc = c_nc[c_nc.size() / 2]; best.bs = 16; best.mfma = mfma;
    best.fuse = cfg.fuse_combine > 0 ? 1 : 0;   // not searched by the cost model: chosen by the caller or by on-device tuning
    best.att_mc = mfma ? 1 : 0;   // (the kernels of the matrix-core path carry only the matrix-core form of the attention task)
    best.page_bytes = kChunkBytes;                      // one page = one 1 KB chunk slot
    // weight-page ring: a pipeline stage is 16 pages (4 per wavefront).  The depth is only searched
    // when asked for (ring_kb == -2): measured on MI355X the direct-load path is the faster one at
    // every depth that fits, so "auto" (-1) keeps weights out of LDS.
    std::vector<int> c_ring;
    if (cfg.ring_kb > 0) c_ring = {cfg.ring_kb / 16 * 16};
    else if (cfg.ring_kb == -2) c_ring = {0, 32, 48, 64, 80, 96, 112, 128};
    else c_ring = {0};
    best.ring_pages = c_ring[0];
    best.n_stage = best.ring_pages ? best.ring_pages / 16 : 1;
    int tried = 0, pruned = 0;
    double best_ms = -1, best_duty = 0;
    auto eval = [&](const Tiling &t, double &ms, double &duty) {
        ++tried;
        if (!admissible(t)) { ++pruned; return false; }
        mk_schedule tmp{};
        int r = assemble(cfg, d, t, &tmp);
        if (r != MK_OK) { ++pruned; return false; }
        ms = tmp.sim.makespan_us; duty = tmp.sim.duty;
        return true;
    };
    struct Dim { int Tiling::*field; std::vector<int> *vals; };
    Dim dimsv[] = {{&Tiling::r_qkv, &c_rq}, {&Tiling::s_qkv, &c_sqkv}, {&Tiling::r_o, &c_ro}, {&Tiling::s_o, &c_so},
                   {&Tiling::r_gu, &c_rgu}, {&Tiling::s_gu, &c_sgu}, {&Tiling::r_d, &c_rd}, {&Tiling::s_d, &c_sd},
                   {&Tiling::nc, &c_nc}, {&Tiling::ring_pages, &c_ring}};
    {
        double ms, du;
        if (eval(best, ms, du)) { best_ms = ms; best_duty = du; }
    }
    for (int round = 0; round < 2; ++round)
        for (auto &dm : dimsv) {
            if (dm.vals->size() < 2 && best_ms >= 0) continue;
            for (int v : *dm.vals) {
                Tiling t = best;
                t.*(dm.field) = v;
                t.n_stage = t.ring_pages ? t.ring_pages / 16 : 1;
                if (t.*(dm.field) == best.*(dm.field) && best_ms >= 0) continue;
                double ms, du;
                if (!eval(t, ms, du)) continue;
                if (best_ms < 0 || ms < best_ms - 1e-9 || (std::fabs(ms - best_ms) <= 1e-9 && du > best_duty)) {
                    best = t; best_ms = ms; best_duty = du;
                }
            }
        }
    if (best_ms < 0) { set_error("no tiling candidate is admissible and fits the LDS budget"); return MK_EINFEASIBLE; }

    mk_schedule *s = new mk_schedule{};
    rc = assemble(cfg, d, best, s);
    if (rc != MK_OK) { delete s; set_error("assembling the chosen candidate failed"); return rc; }
    s->cand_tried = tried; s->cand_pruned = pruned;
    rc = verify_schedule(s);
    if (rc != MK_OK) { delete s; return rc; }
    *out = s;
    return MK_OK;
}

// ---------------------------------------------------------------- verifier
namespace {
struct Access { uint32_t lo, hi; bool write; };

// Memory footprint of one task on the activation region, derived from the instruction alone.
void decode_accesses(const mk_schedule *s, const Instr &I, std::vector<Access> &out)
{
    const Dims &d = s->dm;
    out.clear();
    auto rd = [&](uint64_t lo, uint64_t n) { if (n) out.push_back({(uint32_t)lo, (uint32_t)(lo + n), false}); };
    auto wr = [&](uint64_t lo, uint64_t n) { if (n) out.push_back({(uint32_t)lo, (uint32_t)(lo + n), true}); };
    if (I.op == OP_GEMV) {
        const uint32_t pro = instr_pro(I), np = instr_nparts(I), rlog = instr_rlog(I), R = 1u << rlog, ck = instr_ck(I);
        if (!(I.flags & F_SKIP_PRO)) {
            for (int b = 0; b < d.Bm; ++b) {
                if (pro == PRO_RESID_NORM) {
                    rd(I.in_base + (uint64_t)b * I.in_ld, d.H);
                    for (uint32_t p = 0; p < np; ++p) rd(I.in_parts + (uint64_t)p * I.part_stride + (uint64_t)b * I.in_ld, d.H);
                } else if (pro == PRO_COMBINE) {
                    uint64_t k0 = (uint64_t)I.xs_lo * ck, k1 = std::min<uint64_t>(k0 + (uint64_t)I.xs_hi * ck, I.k_len);
                    const uint64_t h0 = k0 / d.d, nh = (k1 - k0 + d.d - 1) / d.d, RS = d.d + kPartPad;
                    // (the pad words of a row are loaded too but never used, and nobody writes them)
                    for (uint64_t r = 0; k1 > k0 && r < nh * np; ++r) rd(I.in_parts + (((uint64_t)b * d.nq + h0) * np + r) * RS, d.d + 2);
                } else if (pro == PRO_PLAIN || pro == PRO_SILU) {
                    uint64_t k0 = (uint64_t)I.xs_lo * ck, k1 = std::min<uint64_t>(k0 + (uint64_t)I.xs_hi * ck, I.k_len);
                    if (k1 > k0) {
                        uint64_t lo = k0, n = (k1 - k0 + 3) / 4 * 4;
                        if (pro == PRO_SILU) {
                            const uint64_t PR = 1ull << instr_prod_rlog(I), half = PR / 2;
                            lo = (k0 / half) * PR; n = (k1 + half - 1) / half * PR - lo;
                        }
                        for (uint32_t p = 0; p < np; ++p) rd(I.in_parts + (uint64_t)p * I.part_stride + (uint64_t)b * I.in_ld + lo, n);
                    }
                }
                if ((pro == PRO_RESID_NORM || pro == PRO_EMBED_NORM) && I.xs_hi > I.xs_lo)
                    wr(I.xs_out + (uint64_t)b * I.in_ld + I.xs_lo, I.xs_hi - I.xs_lo);
            }
        }
        if (I.flags & F_ARGMAX) wr(s->am.amax + (uint64_t)I.spare * d.Bm * 2, (uint64_t)d.Bm * 2);
        if (!(I.flags & F_LOGITS)) {
            for (uint32_t u = I.u0; u < I.u0 + I.nu; ++u)
                for (int b = 0; b < d.Bm; ++b) {
                    if (I.flags & F_SILU_EPI) {
                        wr(I.out + (uint64_t)b * I.out_ld + (uint64_t)u * (R / 2), R / 2);
                    } else {
                        uint32_t rg, sl;
                        unit_place((I.flags & F_SLICE_MAJOR) != 0, u, I.S, instr_groups(I), rg, sl);
                        const uint64_t row0 = (uint64_t)rg * R;
                        if (I.flags & F_ADD_RESID) rd(I.resid + (uint64_t)b * I.out_ld + row0, R);
                        wr(I.out + (uint64_t)sl * I.out_split_stride + (uint64_t)b * I.out_ld + row0, R);
                    }
                }
        }
    } else if (I.op == OP_RSUM) {
        const uint64_t n = I.xs_hi > I.xs_lo ? I.xs_hi - I.xs_lo : 0;
        for (int b = 0; b < d.Bm; ++b) {
            const uint64_t off = (uint64_t)b * I.in_ld + I.xs_lo;
            rd(I.in_base + off, n);
            for (uint32_t p = 0; p < instr_nparts(I); ++p) rd(I.in_parts + (uint64_t)p * I.part_stride + off, n);
            wr(I.xs_out + off, n);
        }
    } else if (I.op == OP_ATT) {
        const InstrAtt &A = *(const InstrAtt *)&I;
        for (uint32_t p = 0; p < A.n_parts; ++p) {
            uint64_t base = A.in_parts + (uint64_t)p * A.part_stride + (uint64_t)A.b * A.in_ld;
            rd(base + ((uint64_t)A.g * d.G + A.h0) * d.d, (uint64_t)A.nh * d.d);
            rd(base + d.qd + (uint64_t)A.g * d.d, d.d);
            rd(base + d.qd + d.kvd + (uint64_t)A.g * d.d, d.d);
        }
        for (uint32_t h = A.h0; h < A.h0 + A.nh; ++h)
            wr(A.out + (((uint64_t)A.b * d.nq + A.g * d.G + h) * A.nc + A.c) * (d.d + kPartPad), d.d + 2);
    } else if (I.op == OP_COMB) {
        const InstrAtt &A = *(const InstrAtt *)&I;
        for (uint32_t h = A.h0; h < A.h0 + A.nh; ++h) {
            for (uint32_t c = 0; c < A.nc; ++c) rd(A.out + (((uint64_t)A.b * d.nq + h) * A.nc + c) * (d.d + kPartPad), d.d + 2);
            wr(A.o_out + (uint64_t)A.b * A.o_ld + (uint64_t)h * d.d, d.d);
        }
    } else if (I.op == OP_ARGMAX) {
        const InstrAtt &A = *(const InstrAtt *)&I;
        rd(A.out, (uint64_t)A.n_slots * d.Bm * 2);   // every slot's row of every sequence (a superset of what it reads)
    }
}
}  // namespace

int verify_schedule(const mk_schedule *s)
{
    if (!s) { set_error("null schedule"); return MK_EINVAL; }
    char buf[256];
    auto fail = [&](const std::string &m) { set_error("schedule verification failed: " + m); return MK_ESCHED; };
    const int n_wg = s->n_wg, mi = s->max_instr;
    const Dims &d = s->dm;
    const Instr *all = (const Instr *)s->instr.data();
    if (n_wg < 1 || n_wg > 65535 || mi < 1 || (int)s->instr.size() != n_wg * mi * kInstrDwords) return fail("malformed instruction array");
    if (mi > 65535) return fail("instruction list too long");

    // (1) every list ends with END and holds known opcodes; counters: wait target == signals per step
    std::vector<uint32_t> signals(s->n_counters, 0);
    std::vector<int> cnt(n_wg, 0);
    for (int w = 0; w < n_wg; ++w) {
        int i = 0;
        for (; i < mi; ++i) {
            const Instr &I = all[(size_t)w * mi + i];
            if (I.op == OP_END) break;
            if (I.op != OP_GEMV && I.op != OP_ATT && I.op != OP_COMB && I.op != OP_ARGMAX && I.op != OP_RSUM) return fail("unknown opcode");
            if (I.sig_ctr != kNone) {
                if (I.sig_ctr >= (uint32_t)s->n_counters) return fail("signal to a counter that does not exist");
                ++signals[I.sig_ctr];
            }
        }
        if (i == mi) return fail("instruction list without END");
        cnt[w] = i;
    }
    for (int w = 0; w < n_wg; ++w)
        for (int i = 0; i < cnt[w]; ++i) {
            const Instr &I = all[(size_t)w * mi + i];
            for (int k = 0; k < 2; ++k)
                if (I.wait_ctr[k] != kNone) {
                    if (I.wait_ctr[k] >= (uint32_t)s->n_counters) return fail("wait on a counter that does not exist");
                    if (I.wait_cnt[k] != signals[I.wait_ctr[k]]) {
                        snprintf(buf, sizeof buf, "workgroup %d instruction %d waits for %u signals of counter %u, which receives %u",
                                 w, i, I.wait_cnt[k], I.wait_ctr[k], signals[I.wait_ctr[k]]);
                        return fail(buf);
                    }
                }
        }

    // (1b) the fields that address weights, vectors, the KV cache and the attention buffers are not covered
    //      by the activation-footprint walk below: they must equal what the memory maps plan for the
    //      task's (layer, stage), so that a corrupted list cannot reach outside its buffers.
    for (int w = 0; w < n_wg; ++w)
        for (int i = 0; i < cnt[w]; ++i) {
            const Instr &I = all[(size_t)w * mi + i];
            const uint32_t l = I.ref_seq / 8, st = I.ref_seq % 8;
            auto bad = [&](const char *what) {
                snprintf(buf, sizeof buf, "workgroup %d instruction %d (ref_seq %u): %s", w, i, I.ref_seq, what);
                return fail(buf);
            };
            if (I.layer != l) return bad("layer field does not match the operator instance");
            const bool tail = (st == ST_HEAD && I.op != OP_RSUM) || st == ST_ARGMAX;
            if (tail ? l != (uint32_t)d.L : l >= (uint32_t)d.L) return bad("layer out of range");
            if (I.op == OP_RSUM) {
                if (st != ST_RSUM) return bad("residual-sum task at the wrong stage");
                if (!wants_residual_sum(s->tl.s_d, d.Bm, d.H)) return bad("residual-sum task in a schedule that has none");
                const bool ab = I.in_base == s->am.xa && I.xs_out == s->am.xb, ba = I.in_base == s->am.xb && I.xs_out == s->am.xa;
                if (!ab && !ba) return bad("residual buffers differ from the plan");
                if (I.in_parts != s->am.pd || instr_nparts(I) != (uint32_t)s->tl.s_d || I.part_stride != (uint32_t)(d.Bm * d.H) ||
                    I.in_ld != (uint32_t)d.H)
                    return bad("partial-row description differs from the plan");
                if ((I.xs_lo | I.xs_hi) & 3u || I.xs_lo >= I.xs_hi || I.xs_hi > (uint32_t)d.H) return bad("residual slice out of range");
            } else if (I.op == OP_GEMV) {
                const MatGeom *m = nullptr;
                uint32_t chunk = 0, gain = kNone, bias = kNone;
                int S = 1;
                switch (st) {
                case ST_QKV: m = &s->gm.qkv; chunk = s->wm.qkv[l]; S = s->tl.s_qkv; gain = s->wm.g_attn[l]; bias = s->wm.bias[l]; break;
                case ST_O: m = &s->gm.o; chunk = s->wm.o[l]; S = s->tl.s_o; break;
                case ST_GU: m = &s->gm.gu; chunk = s->wm.gu[l]; S = s->tl.s_gu; gain = s->wm.g_mlp[l]; break;
                case ST_DOWN: m = &s->gm.down; chunk = s->wm.down[l]; S = s->tl.s_d; break;
                case ST_HEAD: m = &s->gm.head; chunk = s->wm.head; S = 1; gain = s->wm.g_final; break;
                default: return bad("a GEMV task at a stage that has none");
                }
                if (I.w_chunk != chunk) return bad("weight chunk offset differs from the planned matrix");
                if (I.kbt != (uint32_t)m->kbt || I.S != (uint32_t)S || I.nkb != (uint32_t)ceil_div(m->kbt, S) ||
                    instr_rlog(I) != (uint32_t)m->rlog || I.n_rows != (uint32_t)m->n_rows || I.k_len != (uint32_t)m->k_len ||
                    ((I.flags & F_W4) != 0) != (m->w4 != 0) || ((I.flags & F_MFMA) != 0) != (s->tl.mfma != 0) ||
                    ((I.flags & F_SLICE_MAJOR) != 0) != (m->sm != 0) || instr_groups(I) != (uint32_t)m->groups)
                    return bad("matrix geometry differs from the planned matrix");
                const uint32_t pro = instr_pro(I);
                const bool normk = pro == PRO_EMBED_NORM || pro == PRO_RESID_NORM;
                if (normk != (gain != kNone)) return bad("prologue kind does not fit the operator");
                if (normk && I.gain != gain) return bad("norm gain offset differs from the planned vector");
                if (I.bias != bias) return bad("bias offset differs from the planned vector");
                if ((uint64_t)I.u0 + I.nu > (uint64_t)m->groups * S) return bad("units beyond the matrix");
                if (!normk) {
                    // the staged chunk range must hold the K slice of every unit of the task
                    for (uint32_t u = I.u0; u < I.u0 + I.nu; ++u) {
                        uint32_t rg, sl;
                        unit_place(m->sm != 0, u, I.S, (uint32_t)m->groups, rg, sl);
                        const uint32_t lo = sl * I.nkb, hi = lo + slice_chunks(sl, I.S, I.nkb, I.kbt);
                        if (lo < I.xs_lo || hi > I.xs_lo + I.xs_hi) return bad("a unit's K slice lies outside the staged input range");
                    }
                }
            } else if (I.op == OP_ATT || I.op == OP_COMB) {
                const InstrAtt &A = *(const InstrAtt *)&I;
                if (st != (I.op == OP_ATT ? ST_ATT : ST_COMB)) return bad("attention task at the wrong stage");
                if (A.b >= (uint32_t)d.Bm) return bad("sequence index beyond max_batch");
                if (A.nc != (uint32_t)s->tl.nc) return bad("chunk count differs from the tiling");
                if (A.out != s->am.attp) return bad("attention partial buffer offset differs from the plan");
                if (I.op == OP_ATT) {
                    if (((I.flags & F_ATT_MC) != 0) != (s->tl.att_mc != 0)) return bad("attention form differs from the tiling");
                    if (A.g >= (uint32_t)d.nkv) return bad("kv head out of range");
                    if (A.c >= A.nc) return bad("chunk index out of range");
                    if (A.bs != (uint32_t)s->tl.bs || A.bs != 16u) return bad("block size differs from the tiling");
                    if (A.in_parts != s->am.pqkv || A.n_parts != (uint32_t)s->tl.s_qkv || A.in_ld != (uint32_t)d.nqkv ||
                        A.part_stride != (uint32_t)(d.Bm * d.nqkv))
                        return bad("QKV input description differs from the plan");
                    if (A.qn_gain != s->wm.qn[l] || A.kn_gain != s->wm.kn[l]) return bad("q/k norm gain offset differs from the planned vector");
                } else {
                    if (A.nh == 0 || (uint64_t)A.h0 + A.nh > (uint64_t)d.nq) return bad("combine task with an empty or out-of-range head range");
                    if (A.o_out != s->am.o || A.o_ld != (uint32_t)d.qd) return bad("attention output description differs from the plan");
                }
            } else {   // OP_ARGMAX
                const InstrAtt &A = *(const InstrAtt *)&I;
                if (st != ST_ARGMAX) return bad("arg-max task at the wrong stage");
                if (A.b >= (uint32_t)d.Bm) return bad("sequence index beyond max_batch");
                if (A.out != s->am.amax) return bad("arg-max partial buffer offset differs from the plan");
            }
        }

    // (2) every tile of every operator exactly once
    {
        std::map<uint32_t, std::vector<std::pair<uint32_t, uint32_t>>> units;   // ref_seq -> [u0, u1)
        std::map<uint32_t, std::vector<uint32_t>> keys;
        std::map<uint32_t, uint64_t> att_heads;   // heads covered by the attention tasks of an operator instance
        std::vector<uint32_t> slots, argmax_slots;
        for (int w = 0; w < n_wg; ++w)
            for (int i = 0; i < cnt[w]; ++i) {
                const Instr &I = all[(size_t)w * mi + i];
                if (I.op == OP_GEMV) {
                    if (I.nu == 0 || I.S == 0 || I.nkb == 0) return fail("empty GEMV task");
                    units[I.ref_seq].push_back({I.u0, I.u0 + I.nu});
                    if (I.flags & F_ARGMAX) slots.push_back(I.spare);
                } else if (I.op == OP_RSUM) {
                    units[I.ref_seq].push_back({I.xs_lo, I.xs_hi});   // (slices of the hidden dimension)
                } else {
                    const InstrAtt &A = *(const InstrAtt *)&I;
                    if (I.op == OP_ATT && (A.nh == 0 || A.h0 + A.nh > (uint32_t)d.G)) return fail("attention task with an empty or out-of-group head range");
                    keys[I.ref_seq].push_back(I.op == OP_ATT ? ((A.b * d.nkv + A.g) * A.nc + A.c) * d.G + A.h0 : I.op == OP_COMB ? A.b * d.nq + A.h0 : A.b);
                    if (I.op == OP_ATT) att_heads[I.ref_seq] += A.nh;
                    if (I.op == OP_ARGMAX) argmax_slots.push_back(A.n_slots);
                }
            }
        // arg-max: one task per sequence, the LM-head tasks own the partial slots 0 .. n-1, one each
        {
            auto &v = keys[d.L * 8 + ST_ARGMAX];
            std::sort(v.begin(), v.end());
            if ((int)v.size() != d.Bm) return fail("the step does not end with one arg-max task per sequence");
            for (int b = 0; b < d.Bm; ++b) if (v[b] != (uint32_t)b) return fail("arg-max task missing or duplicated");
            std::sort(slots.begin(), slots.end());
            for (size_t i = 0; i < slots.size(); ++i) if (slots[i] != i) return fail("arg-max partial slot missing or duplicated");
            if (slots.size() > (size_t)s->gm.head.groups) return fail("more arg-max partial slots than the buffer holds");
            for (uint32_t n : argmax_slots) if (n != slots.size()) return fail("arg-max task reduces the wrong number of partial slots");
        }
        for (int l = 0; l <= d.L; ++l) {
            const Geom &gm = s->gm;
            struct { uint32_t st; uint32_t total; } g[] = {
                {ST_QKV, (uint32_t)gm.qkv.groups * s->tl.s_qkv}, {ST_O, (uint32_t)gm.o.groups * s->tl.s_o},
                {ST_GU, (uint32_t)gm.gu.groups * s->tl.s_gu}, {ST_DOWN, (uint32_t)gm.down.groups * s->tl.s_d},
                {ST_HEAD, (uint32_t)gm.head.groups}};
            if (l < d.L) {   // (stage 6 inside a layer: the residual-sum slices tile the hidden dimension, or there are none)
                g[4].st = ST_RSUM;
                g[4].total = wants_residual_sum(s->tl.s_d, d.Bm, d.H) ? (uint32_t)d.H : 0u;
            }
            for (auto &e : g) {
                if (l == d.L && e.st != ST_HEAD) continue;
                auto &v = units[l * 8 + e.st];
                std::sort(v.begin(), v.end());
                uint32_t at = 0;
                for (auto &r : v) {
                    if (r.first != at) { snprintf(buf, sizeof buf, "operator %u of layer %d: unit %u missing or duplicated", e.st, l, at); return fail(buf); }
                    at = r.second;
                }
                if (at != e.total) { snprintf(buf, sizeof buf, "operator %u of layer %d covers %u of %u units", e.st, l, at, e.total); return fail(buf); }
            }
            if (l < d.L) {
                // attention: the head ranges of the tasks of every (sequence, kv head, chunk) tile the group
                // exactly (distinct first heads, d.G heads in all: the write-overlap check below rules out overlaps)
                {
                    auto &v = keys[l * 8 + ST_ATT];
                    std::sort(v.begin(), v.end());
                    if (std::adjacent_find(v.begin(), v.end()) != v.end()) return fail("attention task missing or duplicated");
                    const uint64_t want = (uint64_t)d.Bm * d.nkv * s->tl.nc * d.G;
                    if (att_heads[l * 8 + ST_ATT] != want) { snprintf(buf, sizeof buf, "attention of layer %d covers %llu of %llu (chunk, head) pairs", l, (unsigned long long)att_heads[l * 8 + ST_ATT], (unsigned long long)want); return fail(buf); }
                }
                struct { uint32_t st; uint32_t total; } k2[] = {{ST_COMB, (uint32_t)(s->tl.fuse ? 0 : d.Bm * d.nq)}};
                for (auto &e : k2) {
                    auto &v = keys[l * 8 + e.st];
                    std::sort(v.begin(), v.end());
                    if (v.size() != e.total) { snprintf(buf, sizeof buf, "operator %u of layer %d has %zu of %u tasks", e.st, l, v.size(), e.total); return fail(buf); }
                    for (uint32_t i = 0; i < e.total; ++i) if (v[i] != i) return fail("attention task missing or duplicated");
                }
            }
        }
    }

    // (3) replay with blocking waits: terminates, and yields happens-before vector clocks.
    //     vc[task][w] = number of leading instructions of workgroup w that happen before the task starts.
    std::vector<size_t> first(n_wg + 1, 0);
    for (int w = 0; w < n_wg; ++w) first[w + 1] = first[w] + cnt[w];
    const size_t n_tasks = first[n_wg];
    std::vector<uint16_t> vc(n_tasks * n_wg, 0);
    std::vector<uint16_t> cvc((size_t)s->n_counters * n_wg, 0);
    std::string why;
    bool ok = replay(s, [&](int w, int i, const Instr &I) {
        uint16_t *me = vc.data() + (first[w] + i) * n_wg;
        if (i > 0) memcpy(me, vc.data() + (first[w] + i - 1) * n_wg, sizeof(uint16_t) * n_wg);
        me[w] = (uint16_t)i;
        for (int k = 0; k < 2; ++k)
            if (I.wait_ctr[k] != kNone && !(k == 0 && (I.flags & F_WAIT_PREV))) {
                const uint16_t *c = cvc.data() + (size_t)I.wait_ctr[k] * n_wg;
                for (int x = 0; x < n_wg; ++x) me[x] = std::max(me[x], c[x]);
            }
        if (I.sig_ctr != kNone) {
            uint16_t *c = cvc.data() + (size_t)I.sig_ctr * n_wg;
            for (int x = 0; x < n_wg; ++x) c[x] = std::max(c[x], me[x]);
            c[w] = std::max<uint16_t>(c[w], (uint16_t)(i + 1));
        }
    }, &why);
    if (!ok) return fail(why.empty() ? "replay did not terminate" : why);
    std::vector<uint16_t> t_wg(n_tasks), t_idx(n_tasks);
    for (int w = 0; w < n_wg; ++w)
        for (int i = 0; i < cnt[w]; ++i) { t_wg[first[w] + i] = (uint16_t)w; t_idx[first[w] + i] = (uint16_t)i; }
    auto hb = [&](uint32_t a, uint32_t b) {   // task ids: does a happen before b?
        const int wa = t_wg[a], wb = t_wg[b];
        if (wa == wb) return t_idx[a] < t_idx[b];
        return vc[(size_t)b * n_wg + wa] >= (uint16_t)(t_idx[a] + 1);
    };

    // (3b) steps of a multi-step launch follow each other without a kernel boundary.  They stay
    //      ordered because (i) every task waits on something, (ii) only the first operator of a step
    //      waits at the previous step's target, and it waits for the arg-max counter, (iii) every
    //      task of a step happens before one of the arg-max tasks that signal that counter: so no
    //      task of step e+1 starts before every task of step e has drained its stores.
    {
        std::vector<uint32_t> amx;
        uint32_t amx_ctr = kNone;
        for (uint32_t t = 0; t < n_tasks; ++t) {
            const Instr &I = all[(size_t)t_wg[t] * mi + t_idx[t]];
            if (I.op == OP_ARGMAX) { amx.push_back(t); amx_ctr = I.sig_ctr; }
        }
        for (uint32_t t = 0; t < n_tasks; ++t) {
            const Instr &I = all[(size_t)t_wg[t] * mi + t_idx[t]];
            if (I.wait_ctr[0] == kNone) return fail("a task waits on nothing: steps of one launch could overlap");
            if (I.flags & F_WAIT_PREV) {
                if (I.op != OP_GEMV || I.ref_seq != ST_QKV || I.wait_ctr[0] != amx_ctr) return fail("only the first operator may wait for the previous step, and only on the arg-max counter");
            } else if (I.op == OP_GEMV && I.ref_seq == ST_QKV) {
                return fail("the first operator of a step must wait for the previous step's arg-max");
            }
            if (I.op == OP_ARGMAX) continue;
            bool before = false;
            for (uint32_t a : amx) before = before || hb(t, a);
            if (!before) { snprintf(buf, sizeof buf, "task ref_seq %u is not ordered before the arg-max that closes the step", I.ref_seq); return fail(buf); }
        }
    }

    // (4) walk the tasks in topological (operator) order with a last-writers table: every
    //     read-after-write, write-after-read and write-after-write pair must be ordered.
    std::vector<uint32_t> order(n_tasks);
    std::iota(order.begin(), order.end(), 0u);
    auto instr_of = [&](uint32_t t) -> const Instr & { return all[(size_t)t_wg[t] * mi + t_idx[t]]; };
    std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return instr_of(a).ref_seq < instr_of(b).ref_seq; });
    // F_SKIP_PRO is only legal directly after a GEMV of the same operator instance with the same staged input
    for (int w = 0; w < n_wg; ++w)
        for (int i = 0; i < cnt[w]; ++i) {
            const Instr &I = all[(size_t)w * mi + i];
            if (I.op == OP_GEMV && (I.flags & F_SKIP_PRO)) {
                if (i == 0) return fail("first instruction skips its prologue");
                const Instr &Pv = all[(size_t)w * mi + i - 1];
                bool same = Pv.op == OP_GEMV && Pv.ref_seq == I.ref_seq && Pv.cfg == I.cfg;
                if (same && (instr_pro(I) == PRO_PLAIN || instr_pro(I) == PRO_SILU || instr_pro(I) == PRO_COMBINE)) same = Pv.xs_lo == I.xs_lo && Pv.xs_hi == I.xs_hi;
                if (!same) return fail("prologue skipped although LDS does not hold this task's input");
            }
        }
    const uint32_t BK = 256;                                   // floats per bucket
    const size_t n_b = (s->am.n_floats + BK - 1) / BK + 1;
    struct Rec { uint32_t lo, hi, task; };
    std::vector<std::vector<Rec>> reads(n_b);
    std::map<uint32_t, Rec> writers;                           // lo -> non-overlapping last-writer intervals
    std::vector<Access> acc;
    for (uint32_t t : order) {
        const Instr &I = instr_of(t);
        decode_accesses(s, I, acc);
        for (const Access &a : acc) {
            if (a.hi > s->am.n_floats) return fail("task touches memory outside the activation region");
            if (!a.write) {
                // RAW: the whole range must have been written earlier in this step, by tasks ordered before us
                uint32_t at = a.lo;
                auto it = writers.upper_bound(a.lo);
                if (it != writers.begin()) --it;
                for (; it != writers.end() && it->second.lo < a.hi; ++it) {
                    const Rec &r = it->second;
                    if (r.hi <= a.lo) continue;
                    if (r.lo > at) break;
                    if (!hb(r.task, t)) {
                        snprintf(buf, sizeof buf, "read-after-write not ordered: task ref_seq %u reads [%u,%u) written by ref_seq %u",
                                 I.ref_seq, a.lo, a.hi, instr_of(r.task).ref_seq);
                        return fail(buf);
                    }
                    at = std::max(at, r.hi);
                }
                if (at < a.hi) {
                    snprintf(buf, sizeof buf, "task ref_seq %u reads [%u,%u) that no earlier task of the step wrote (from %u)", I.ref_seq, a.lo, a.hi, at);
                    return fail(buf);
                }
                for (size_t bk = a.lo / BK; bk <= (a.hi - 1) / BK; ++bk) reads[bk].push_back({a.lo, a.hi, t});
            } else {
                for (size_t bk = a.lo / BK; bk <= (a.hi - 1) / BK; ++bk)
                    for (const Rec &r : reads[bk])
                        if (r.lo < a.hi && a.lo < r.hi && r.task != t && !hb(r.task, t)) {
                            snprintf(buf, sizeof buf, "write-after-read not ordered: ref_seq %u overwrites [%u,%u) still read by ref_seq %u",
                                     I.ref_seq, a.lo, a.hi, instr_of(r.task).ref_seq);
                            return fail(buf);
                        }
                // WAW against the last writers, then replace them
                auto it = writers.upper_bound(a.lo);
                if (it != writers.begin()) --it;
                std::vector<Rec> keep;
                while (it != writers.end() && it->second.lo < a.hi) {
                    Rec r = it->second;
                    if (r.hi <= a.lo) { ++it; continue; }
                    if (r.task != t && !hb(r.task, t)) {
                        snprintf(buf, sizeof buf, "write-after-write not ordered on [%u,%u): ref_seq %u vs %u", a.lo, a.hi, I.ref_seq, instr_of(r.task).ref_seq);
                        return fail(buf);
                    }
                    if (r.lo < a.lo) keep.push_back({r.lo, a.lo, r.task});
                    if (r.hi > a.hi) keep.push_back({a.hi, r.hi, r.task});
                    it = writers.erase(it);
                }
                for (auto &k : keep) writers[k.lo] = k;
                writers[a.lo] = {a.lo, a.hi, t};
            }
        }
    }
    return MK_OK;
}

// ---------------------------------------------------------------- serialisation
namespace {
struct BlobHeader {
    uint32_t magic, version;
    mk_config cfg;
    Tiling tl;
    int32_t n_wg, max_instr, n_counters, n_tasks;
    uint32_t lds_red_bytes, lds_xs_off, lds_total;
    double sim_makespan, sim_duty;
    int32_t cand_tried, cand_pruned;
    uint64_t n_instr_words;
};
constexpr uint32_t kMagic = 0x4d4b5343u;  // "MKSC"
constexpr uint32_t kVersion = 7;
}  // namespace

int dump_schedule(const mk_schedule *s, void *buf, size_t *bytes)
{
    if (!s || !bytes) { set_error("null argument"); return MK_EINVAL; }
    size_t need = sizeof(BlobHeader) + s->instr.size() * 4;
    if (!buf) { *bytes = need; return MK_OK; }
    if (*bytes < need) { *bytes = need; set_error("dump buffer too small"); return MK_ENOMEM; }
    BlobHeader h{};
    h.magic = kMagic; h.version = kVersion; h.cfg = s->cfg; h.tl = s->tl;
    h.n_wg = s->n_wg; h.max_instr = s->max_instr; h.n_counters = s->n_counters; h.n_tasks = s->n_tasks;
    h.lds_red_bytes = s->lds_red_bytes; h.lds_xs_off = s->lds_xs_off; h.lds_total = s->lds_total;
    h.sim_makespan = s->sim.makespan_us; h.sim_duty = s->sim.duty;
    h.cand_tried = s->cand_tried; h.cand_pruned = s->cand_pruned;
    h.n_instr_words = s->instr.size();
    memcpy(buf, &h, sizeof h);
    memcpy((char *)buf + sizeof h, s->instr.data(), s->instr.size() * 4);
    *bytes = need;
    return MK_OK;
}

int load_schedule(const void *buf, size_t bytes, mk_schedule **out)
{
    if (!buf || !out || bytes < sizeof(BlobHeader)) { set_error("blob too small"); return MK_EINVAL; }
    BlobHeader h;
    memcpy(&h, buf, sizeof h);
    if (h.magic != kMagic || h.version != kVersion) { set_error("not a schedule blob of this version"); return MK_EINVAL; }
    if (bytes != sizeof h + h.n_instr_words * 4 || h.n_wg < 1 || h.max_instr < 1 ||
        h.n_instr_words != (uint64_t)h.n_wg * h.max_instr * kInstrDwords) { set_error("truncated or inconsistent schedule blob"); return MK_EINVAL; }
    Dims d;
    mk_config cfg = h.cfg;
    if (cfg.n_workgroups != h.n_wg) { set_error("schedule blob: workgroup count mismatch"); return MK_EINVAL; }
    int rc = derive_dims(cfg, d);
    if (rc) return rc;
    // rebuild the memory maps from the stored tiling, then take the stored instruction lists
    mk_schedule *s = new mk_schedule{};
    rc = assemble(cfg, d, h.tl, s);
    if (rc != MK_OK) { delete s; set_error("schedule blob: stored tiling does not assemble"); return rc; }
    if (s->max_instr != h.max_instr || s->n_counters != h.n_counters) { delete s; set_error("schedule blob: layout mismatch"); return MK_EINVAL; }
    memcpy(s->instr.data(), (const char *)buf + sizeof h, h.n_instr_words * 4);
    s->cand_tried = h.cand_tried; s->cand_pruned = h.cand_pruned;
    rc = verify_schedule(s);
    if (rc != MK_OK) { delete s; return rc; }
    *out = s;
    return MK_OK;
}

}  // namespace mk
