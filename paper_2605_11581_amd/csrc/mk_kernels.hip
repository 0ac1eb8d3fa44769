// CDNA4 (gfx950) device code of the decode-step megakernel.
//
// One persistent launch (mk_megakernel) walks a static per-workgroup
// instruction list (paper Sec. 4.2.2 Step 4): each instruction is one
// tile-task of the decoder DAG -- a contiguous run of 1 KB weight chunks of a
// GEMV, a slice of the KV cache for flash-decode attention, or a partial
// combine.  Dependencies are global-memory counters with per-step epoch
// targets; nothing is decided at run time.  The per-operator baseline
// (mk_op_kernel) runs the same task bodies, one launch per DAG operator.
//
// Weight streaming follows the paper's decoupling (Sec. 4.2.3, Fig. 4): loads
// that do not depend on the previous operator (the task's first weight chunks)
// are issued before the dependency wait.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mk_isa.h"

namespace mk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct LdsPlan {
    uint32_t red_bytes;   // cross-wave reduction region
    uint32_t xs_off;      // byte offset of the staged-input region
};

// ---------------------------------------------------------------- small helpers
__device__ __forceinline__ uint32_t rfl(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf_to_f(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// fp32 -> bf16, round to nearest even (finite inputs; NaN kept quiet)
__device__ __forceinline__ uint16_t f_to_bf(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ void set_err(const Params &P, int slot, uint32_t v)
{
    uint32_t *e = (uint32_t *)(P.ws + P.lay.err);
    __hip_atomic_store(e + slot, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Poll a dependency counter until it has received `target` signals (wrap-safe).
// Bounded: after `limit` polls the wait gives up and reports failure, so every
// wave always reaches the end of its instruction list.
__device__ __forceinline__ bool wait_counter(const uint32_t *ctr, uint32_t target, uint32_t limit)
{
    uint32_t it = 0;
    while ((int32_t)(__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
        __builtin_amdgcn_s_sleep(1);
        if (++it > limit) return false;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // later loads see the producers' stores
    return true;
}

__device__ __forceinline__ int clamp_i(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

__device__ __forceinline__ int token_of(const Params &P, int b)
{
    int t = P.tokens[b];
    if (t < 0 || t >= P.vocab) { set_err(P, 1, 1u); t = clamp_i(t, 0, P.vocab - 1); }
    return t;
}
__device__ __forceinline__ int position_of(const Params &P, int b)
{
    int p = P.positions[b];
    if (p < 0 || p >= P.max_context) { set_err(P, 1, 2u); p = clamp_i(p, 0, P.max_context - 1); }
    return p;
}

// Element (row, k) of a tile-major matrix whose first chunk is `chunk0`.
__device__ __forceinline__ float tile_elem(const char *wbase, uint32_t chunk0, uint32_t kbt, int row, int k)
{
    size_t chunk = (size_t)chunk0 + (size_t)(row >> 4) * kbt + (size_t)(k >> 5);
    int slot = ((k & 31) >> 3) * 16 + (row & 15);
    const uint16_t *p = (const uint16_t *)(wbase + chunk * kChunkBytes + slot * 16) + (k & 7);
    return bf_to_f(*p);
}

// ---------------------------------------------------------------- GEMV task
// Staged input in LDS:
//   VALU path (batch 1): fp32 x[k]
//   MFMA path: bf16 planes [col][k], col = b * nterm + term, x = sum of its nterm bf16 terms;
//              plane stride = k_stage * 2 + 16 bytes (bank skew)
template <bool MFMA>
__device__ __forceinline__ void store_x(char *xs, int b, int i, float y, int nterm, uint32_t plane_stride)
{
    if (!MFMA) {
        ((float *)xs)[i] = y;
    } else {
        float r = y;
        for (int t = 0; t < nterm; ++t) {
            uint16_t h = f_to_bf(r);
            *(uint16_t *)(xs + (size_t)(b * nterm + t) * plane_stride + (size_t)i * 2) = h;
            r -= bf_to_f(h);
        }
    }
}

__device__ __forceinline__ int nterm_of(int batch) { return batch <= 5 ? 3 : 2; }

template <bool MFMA>
__device__ void gemv_prologue(const Params &P, const Instr &I, char *lds, const LdsPlan &lp, int batch)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    char *xs = lds + lp.xs_off;
    float *misc = (float *)(lds + kLdsMisc);
    const float *act = (const float *)(P.ws + P.lay.act);
    float *actw = (float *)(P.ws + P.lay.act);
    const int nterm = nterm_of(batch);
    const uint32_t pro = I.pro;

    if (pro == PRO_EMBED_NORM || pro == PRO_RESID_NORM) {
        const int H = P.hidden;
        const uint32_t plane_stride = (uint32_t)H * 2u + 16u;
        const uint16_t *gain = (const uint16_t *)(P.ws + P.lay.vecs) + I.gain;
        const uint32_t kbtH = (uint32_t)H >> 5;
        for (int b = 0; b < batch; ++b) {
            float v[16];
            float ss = 0.f;
            int tok = 0;
            if (pro == PRO_EMBED_NORM) tok = token_of(P, b);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                int i = tid + j * kWgThreads;
                float x = 0.f;
                if (i < H) {
                    if (pro == PRO_EMBED_NORM) {
                        x = tile_elem(P.ws + P.lay.weights, P.embed_chunk, kbtH, tok, i);
                    } else {
                        x = act[I.in_base + (size_t)b * I.in_ld + i];
                        for (uint32_t s = 0; s < I.n_parts; ++s)
                            x += act[I.in_parts + (size_t)s * I.part_stride + (size_t)b * I.in_ld + i];
                    }
                    if ((uint32_t)i >= I.xs_lo && (uint32_t)i < I.xs_hi) actw[I.xs_out + (size_t)b * I.in_ld + i] = x;
                }
                v[j] = x;
                ss += x * x;
            }
            ss = wave_sum(ss);
            float *slot = misc + (b & 1) * 8;
            if (lane == 0) slot[wave] = ss;
            __syncthreads();
            float tot = slot[0] + slot[1] + slot[2] + slot[3];
            float inv = 1.0f / sqrtf(tot / (float)H + P.rms_eps);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                int i = tid + j * kWgThreads;
                if (i < H) store_x<MFMA>(xs, b, i, v[j] * inv * bf_to_f(gain[i]), nterm, plane_stride);
            }
        }
    } else {
        // PLAIN / SILU: stage k blocks [xs_lo, xs_lo + xs_hi) of the input
        const int k0 = (int)I.xs_lo * kChunkK, kn = (int)I.xs_hi * kChunkK;
        const uint32_t plane_stride = (uint32_t)kn * 2u + 16u;
        for (int b = 0; b < batch; ++b) {
            for (int i = tid; i < kn; i += kWgThreads) {
                int k = k0 + i;
                float y = 0.f;
                if ((uint32_t)k < I.k_len) {
                    if (pro == PRO_PLAIN) {
                        for (uint32_t s = 0; s < I.n_parts; ++s)
                            y += act[I.in_parts + (size_t)s * I.part_stride + (size_t)b * I.in_ld + k];
                    } else {
                        size_t gi = (size_t)(k >> 4) * 32 + (k & 15);
                        float gsum = 0.f, usum = 0.f;
                        for (uint32_t s = 0; s < I.n_parts; ++s) {
                            const float *pp = act + I.in_parts + (size_t)s * I.part_stride + (size_t)b * I.in_ld;
                            gsum += pp[gi];
                            usum += pp[gi + 16];
                        }
                        y = gsum / (1.0f + __expf(-gsum)) * usum;
                    }
                }
                store_x<MFMA>(xs, b, i, y, nterm, plane_stride);
            }
        }
    }
    __syncthreads();
}

// k blocks in unit u of a matrix with S splits of nkb blocks per row block (last split ragged)
__device__ __forceinline__ uint32_t unit_nkb(uint32_t u, uint32_t S, uint32_t nkb, uint32_t kbt)
{
    uint32_t s = u % S;
    return (s == S - 1) ? kbt - s * nkb : nkb;
}


struct GemvStream {
    const u32x4 *wp;      // this lane's pointer to chunk 0 of the task
    uint32_t total;       // chunks in the task
    u32x4 buf[kPrefetch];
};

// Issue the first weight loads of a GEMV task.  They depend on nothing the
// previous operator produces, so this runs before the dependency wait.
__device__ __forceinline__ void gemv_issue(const Params &P, const Instr &I, GemvStream &st)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t first = (I.u0 / I.S) * I.kbt + (I.u0 % I.S) * I.nkb;
    uint32_t ulast = I.u0 + I.nu;  // one past the last unit
    uint32_t end = (ulast / I.S) * I.kbt + (ulast % I.S) * I.nkb;
    st.total = end - first;
    st.wp = (const u32x4 *)(P.ws + P.lay.weights) + ((size_t)I.w_chunk + first) * 64 + lane;
#pragma unroll
    for (int j = 0; j < kPrefetch; ++j) {
        uint32_t idx = (uint32_t)wave + (uint32_t)j * kWaves;
        if (idx < st.total) st.buf[j] = __builtin_nontemporal_load(st.wp + (size_t)idx * 64);
    }
}

template <bool MFMA>
__device__ void gemv_main(const Params &P, const Instr &I, char *lds, const LdsPlan &lp, GemvStream &st, int batch)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ksub = lane >> 4;
    char *xs = lds + lp.xs_off;
    float *red = (float *)(lds + kLdsRed);
    const int nterm = nterm_of(batch);
    const int ncols = MFMA ? batch * nterm : 1;
    const uint32_t S = I.S, nkb = I.nkb, kbt = I.kbt, nu = I.nu, u0 = I.u0;
    const bool normk = (I.pro == PRO_EMBED_NORM || I.pro == PRO_RESID_NORM);
    const uint32_t x_kb0 = normk ? 0u : I.xs_lo;
    const uint32_t k_stage = normk ? (uint32_t)P.hidden : I.xs_hi * kChunkK;
    const uint32_t plane_stride = k_stage * 2u + 16u;
    const uint32_t red_per_wave = nu * 16u * (uint32_t)(MFMA ? batch : 1);

    // running position of this wave inside the task: unit ul, k block kbi within the unit
    uint32_t ul = 0, kbi = (uint32_t)wave;
    uint32_t cur_n = unit_nkb(u0, S, nkb, kbt);
    uint32_t cur_kb0 = (u0 % S) * nkb;  // first k block of the current unit inside its row block

    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    f32x4 cacc = {0.f, 0.f, 0.f, 0.f};

    auto flush = [&]() {
        if (!MFMA) {
            float v = (a0 + a1) + (a2 + a3);
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (lane < 16) red[wave * red_per_wave + ul * 16 + lane] = v;
            a0 = a1 = a2 = a3 = 0.f;
        } else {
            // cacc[j] = C[row 4*ksub + j][col lane & 15]; sum the nterm columns of each sequence
            const int col = lane & 15;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float v = cacc[j];
                float v1 = __shfl_down(v, 1, 64);
                float v2 = __shfl_down(v, 2, 64);
                float sum = v + v1 + (nterm == 3 ? v2 : 0.f);
                int b = col / nterm;
                if (col < ncols && col == b * nterm)
                    red[wave * red_per_wave + (ul * batch + b) * 16 + ksub * 4 + j] = sum;
                cacc[j] = 0.f;
            }
        }
    };

    auto consume = [&](const u32x4 &w) {
        // advance to the unit that holds this chunk, flushing finished units
        while (kbi >= cur_n) {
            kbi -= cur_n;
            flush();
            ++ul;
            cur_n = unit_nkb(u0 + ul, S, nkb, kbt);
            cur_kb0 = ((u0 + ul) % S) * nkb;
        }
        const uint32_t kb_rel = cur_kb0 + kbi - x_kb0;  // k block inside the staged vector
        if (!MFMA) {
            const float4 *xp = (const float4 *)(xs + ((size_t)kb_rel * kChunkK + ksub * 8) * 4);
            float4 x0 = xp[0], x1 = xp[1];
            a0 += bf_lo(w.x) * x0.x; a1 += bf_hi(w.x) * x0.y;
            a2 += bf_lo(w.y) * x0.z; a3 += bf_hi(w.y) * x0.w;
            a0 += bf_lo(w.z) * x1.x; a1 += bf_hi(w.z) * x1.y;
            a2 += bf_lo(w.w) * x1.z; a3 += bf_hi(w.w) * x1.w;
        } else {
            const int col = lane & 15;
            u32x4 xb = {0u, 0u, 0u, 0u};
            if (col < ncols)
                xb = *(const u32x4 *)(xs + (size_t)col * plane_stride + ((size_t)kb_rel * kChunkK + ksub * 8) * 2);
            bf16x8 av = __builtin_bit_cast(bf16x8, w);
            bf16x8 bv = __builtin_bit_cast(bf16x8, xb);
            cacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, cacc, 0, 0, 0);
        }
        kbi += kWaves;
    };

    const uint32_t total = st.total;
    for (uint32_t base = 0; base < total; base += kPrefetch * kWaves) {
#pragma unroll
        for (int j = 0; j < kPrefetch; ++j) {
            uint32_t idx = base + (uint32_t)j * kWaves + (uint32_t)wave;
            if (idx < total) {
                u32x4 w = st.buf[j];
                uint32_t nidx = idx + kPrefetch * kWaves;
                if (nidx < total) st.buf[j] = __builtin_nontemporal_load(st.wp + (size_t)nidx * 64);
                consume(w);
            }
        }
    }
    // flush the current unit and any trailing units this wave had no chunk in
    while (ul < nu) {
        flush();
        ++ul;
    }
    __syncthreads();

    // cross-wave sum in fixed wave order, bias, store
    const uint32_t nout = red_per_wave;
    float *actw = (float *)(P.ws + P.lay.act);
    for (uint32_t t = tid; t < nout; t += kWgThreads) {
        float v = red[t];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) v += red[w * red_per_wave + t];
        uint32_t r = t & 15u, ub = t >> 4;
        uint32_t b = MFMA ? ub % (uint32_t)batch : 0u;
        uint32_t uu = u0 + (MFMA ? ub / (uint32_t)batch : ub);
        uint32_t rb = uu / S, s = uu % S;
        uint32_t row = rb * 16u + r;
        if (I.bias != kNone && s == 0 && row < I.n_rows)
            v += bf_to_f(((const uint16_t *)(P.ws + P.lay.vecs))[I.bias + row]);
        if (I.flags & F_LOGITS) {
            if (row < I.n_rows) P.logits[(size_t)b * P.vocab + row] = v;
        } else {
            actw[I.out + (size_t)s * I.out_split_stride + (size_t)b * I.out_ld + row] = v;
        }
    }
}

// ---------------------------------------------------------------- attention task
// Flash-decode partial over the history positions owned by chunk task c of
// (sequence b, kv head g): blocks c, c+nc, c+2nc, ... of `bs` positions.  All
// q heads of the group are processed against each K/V row read once.  The
// task that owns the block of the current position also rotates/rounds the
// new k and v, appends them to the cache and attends to them from LDS.
struct AttState {
    float m[kMaxGroup], l[kMaxGroup];
    float acc[kMaxGroup][8];
};

__device__ __forceinline__ float safe_exp_diff(float a, float M)
{
    return (a == -INFINITY) ? 0.f : __expf(a - M);
}

template <int D>
__device__ void att_task(const Params &P, const InstrAtt &I, char *lds, const LdsPlan &lp)
{
    constexpr int LPP = D / 8;       // lanes per position (16 B each)
    constexpr int PPW = 64 / LPP;    // positions per wavefront load
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = (int)I.b, g = (int)I.g;
    if (b >= P.batch) return;
    const int G = P.n_q_heads / P.n_kv_heads;
    const int p = position_of(P, b);
    const int qd = P.n_q_heads * D, kvd = P.n_kv_heads * D;
    const float *act = (const float *)(P.ws + P.lay.act);
    const uint16_t *vecs = (const uint16_t *)(P.ws + P.lay.vecs);
    const float *rope = (const float *)(P.ws + P.lay.rope) + (size_t)p * D;  // [D/2][2]

    // LDS scratch inside the xs region
    float *sq = (float *)(lds + lp.xs_off);              // [G][D] rotated, pre-scaled q
    float *snew = sq + kMaxGroup * D;                    // [2][D] new k (rotated, bf16-rounded) and v
    float *smerge = snew + 2 * D;                        // [kWaves][G][D + 2]
    const int jb_new = p / (int)I.bs;
    const bool owner = (jb_new % (int)I.nc) == (int)I.c;

    // ---- prologue: q heads (and new k / v) : sum partials, optional RMSNorm, RoPE
    const int nvec = G + (owner ? 2 : 0);
    for (int vi = wave; vi < nvec; vi += kWaves) {
        int row0;   // first row of this vector in the fused QKV output
        uint32_t gain_off = kNone;
        bool rot = true;
        if (vi < G) { row0 = (g * G + vi) * D; gain_off = I.qn_gain; }
        else if (vi == G) { row0 = qd + g * D; gain_off = I.kn_gain; }
        else { row0 = qd + kvd + g * D; rot = false; }
        const int i = lane;   // pair index (i, i + D/2)
        float a = 0.f, c2 = 0.f;
        if (i < D / 2) {
            for (uint32_t s = 0; s < I.n_parts; ++s) {
                const float *pp = act + I.in_parts + (size_t)s * I.part_stride + (size_t)b * I.in_ld + row0;
                a += pp[i];
                c2 += pp[i + D / 2];
            }
        }
        if (rot) {
            if (P.qk_norm && gain_off != kNone) {
                float ss = wave_sum(a * a + c2 * c2);
                float inv = 1.0f / sqrtf(ss / (float)D + P.rms_eps);
                if (i < D / 2) {
                    a = a * inv * bf_to_f(vecs[gain_off + i]);
                    c2 = c2 * inv * bf_to_f(vecs[gain_off + i + D / 2]);
                }
            }
            if (i < D / 2) {
                float cs = rope[2 * i], sn = rope[2 * i + 1];
                float ra = a * cs - c2 * sn;
                float rb = c2 * cs + a * sn;
                a = ra; c2 = rb;
            }
        }
        if (i < D / 2) {
            if (vi < G) {
                const float scale = 1.0f / sqrtf((float)D);
                sq[vi * D + i] = a * scale;
                sq[vi * D + i + D / 2] = c2 * scale;
            } else {
                const int which = vi - G;  // 0 = K, 1 = V
                uint16_t h0 = f_to_bf(a), h1 = f_to_bf(c2);
                size_t base = ((((size_t)I.layer * 2 + which) * P.max_batch + b) * P.n_kv_heads + g) *
                                  (size_t)P.max_context * D + (size_t)p * D;
                P.kv[base + i] = h0;
                P.kv[base + i + D / 2] = h1;
                snew[which * D + i] = bf_to_f(h0);
                snew[which * D + i + D / 2] = bf_to_f(h1);
            }
        }
    }
    __syncthreads();

    // ---- main loop over this task's history positions (t < p)
    const int sub = lane / LPP, dl = lane % LPP;   // position inside the load, 8-dim slice
    float qr[kMaxGroup][8];
#pragma unroll
    for (int h = 0; h < kMaxGroup; ++h)
        if (h < G) {
            const float4 *qp = (const float4 *)(sq + h * D + dl * 8);
            float4 q0 = qp[0], q1 = qp[1];
            qr[h][0] = q0.x; qr[h][1] = q0.y; qr[h][2] = q0.z; qr[h][3] = q0.w;
            qr[h][4] = q1.x; qr[h][5] = q1.y; qr[h][6] = q1.z; qr[h][7] = q1.w;
        }
    AttState st;
#pragma unroll
    for (int h = 0; h < kMaxGroup; ++h) {
        st.m[h] = -INFINITY; st.l[h] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) st.acc[h][j] = 0.f;
    }
    const size_t head_elems = (size_t)P.max_context * D;
    const uint16_t *Kc = P.kv + ((((size_t)I.layer * 2 + 0) * P.max_batch + b) * P.n_kv_heads + g) * head_elems;
    const uint16_t *Vc = P.kv + ((((size_t)I.layer * 2 + 1) * P.max_batch + b) * P.n_kv_heads + g) * head_elems;
    const int bs = (int)I.bs, nc = (int)I.nc, c = (int)I.c;
    // number of this task's blocks that start before p
    const int nblk_all = (p + bs - 1) / bs;                       // blocks containing positions < p
    const int my_blocks = (nblk_all > c) ? (nblk_all - c + nc - 1) / nc : 0;
    const int npos = my_blocks * bs;                              // flattened (some may be >= p)

    auto step = [&](const u32x4 &kw, const u32x4 &vw, bool valid) {
        float kf[8] = {bf_lo(kw.x), bf_hi(kw.x), bf_lo(kw.y), bf_hi(kw.y), bf_lo(kw.z), bf_hi(kw.z), bf_lo(kw.w), bf_hi(kw.w)};
        float vf[8] = {bf_lo(vw.x), bf_hi(vw.x), bf_lo(vw.y), bf_hi(vw.y), bf_lo(vw.z), bf_hi(vw.z), bf_lo(vw.w), bf_hi(vw.w)};
#pragma unroll
        for (int h = 0; h < kMaxGroup; ++h)
            if (h < G) {
                float s = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) s += qr[h][j] * kf[j];
#pragma unroll
                for (int o = LPP / 2; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
                if (valid) {
                    float mn = fmaxf(st.m[h], s);
                    float sc = safe_exp_diff(st.m[h], mn);
                    float pe = __expf(s - mn);
                    st.l[h] = st.l[h] * sc + pe;
#pragma unroll
                    for (int j = 0; j < 8; ++j) st.acc[h][j] = st.acc[h][j] * sc + pe * vf[j];
                    st.m[h] = mn;
                }
            }
    };

    for (int grp = wave * PPW; grp < npos; grp += kWaves * PPW) {
        int idx = grp + sub;
        int blk = idx / bs;
        int t = (c + blk * nc) * bs + (idx - blk * bs);
        bool valid = t < p;
        u32x4 kw = {0u, 0u, 0u, 0u}, vw = {0u, 0u, 0u, 0u};
        if (valid) {
            kw = __builtin_nontemporal_load((const u32x4 *)(Kc + (size_t)t * D) + dl);
            vw = __builtin_nontemporal_load((const u32x4 *)(Vc + (size_t)t * D) + dl);
        }
        step(kw, vw, valid);
    }
    // the new position, from LDS, by the first position slot of wave 0 of the owner task
    if (owner && wave == 0) {
        const float *kn = snew + dl * 8, *vn = snew + D + dl * 8;
        u32x4 kw, vw;
        kw.x = (uint32_t)f_to_bf(kn[0]) | ((uint32_t)f_to_bf(kn[1]) << 16);
        kw.y = (uint32_t)f_to_bf(kn[2]) | ((uint32_t)f_to_bf(kn[3]) << 16);
        kw.z = (uint32_t)f_to_bf(kn[4]) | ((uint32_t)f_to_bf(kn[5]) << 16);
        kw.w = (uint32_t)f_to_bf(kn[6]) | ((uint32_t)f_to_bf(kn[7]) << 16);
        vw.x = (uint32_t)f_to_bf(vn[0]) | ((uint32_t)f_to_bf(vn[1]) << 16);
        vw.y = (uint32_t)f_to_bf(vn[2]) | ((uint32_t)f_to_bf(vn[3]) << 16);
        vw.z = (uint32_t)f_to_bf(vn[4]) | ((uint32_t)f_to_bf(vn[5]) << 16);
        vw.w = (uint32_t)f_to_bf(vn[6]) | ((uint32_t)f_to_bf(vn[7]) << 16);
        step(kw, vw, sub == 0);
    }

    // ---- merge the PPW position slots of the wave (butterfly over lane bits >= LPP)
#pragma unroll
    for (int o = LPP; o < 64; o <<= 1) {
#pragma unroll
        for (int h = 0; h < kMaxGroup; ++h)
            if (h < G) {
                float mo = __shfl_xor(st.m[h], o, 64), lo = __shfl_xor(st.l[h], o, 64);
                float M = fmaxf(st.m[h], mo);
                float fa = safe_exp_diff(st.m[h], M), fb = safe_exp_diff(mo, M);
                st.l[h] = st.l[h] * fa + lo * fb;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    float ao = __shfl_xor(st.acc[h][j], o, 64);
                    st.acc[h][j] = st.acc[h][j] * fa + ao * fb;
                }
                st.m[h] = M;
            }
    }
    if (sub == 0) {
#pragma unroll
        for (int h = 0; h < kMaxGroup; ++h)
            if (h < G) {
                float *dst = smerge + ((size_t)wave * G + h) * (D + 2);
#pragma unroll
                for (int j = 0; j < 8; ++j) dst[dl * 8 + j] = st.acc[h][j];
                if (dl == 0) { dst[D] = st.m[h]; dst[D + 1] = st.l[h]; }
            }
    }
    __syncthreads();

    // ---- merge the waves in fixed order and write the task's partial
    float *outp = (float *)(P.ws + P.lay.act) + I.out;
    for (int e = tid; e < G * D; e += kWgThreads) {
        int h = e / D, i = e % D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, smerge[((size_t)w * G + h) * (D + 2) + D]);
        float L = 0.f, A = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float *src = smerge + ((size_t)w * G + h) * (D + 2);
            float f = safe_exp_diff(src[D], M);
            L += src[D + 1] * f;
            A += src[i] * f;
        }
        // partial layout [b][head][nc][D + 2]
        float *dst = outp + ((((size_t)b * P.n_q_heads + (g * G + h)) * I.nc) + I.c) * (D + 2);
        dst[i] = A;
        if (i == 0) { dst[D] = M; dst[D + 1] = L; }
    }
}

// Combine the nc flash-decode partials of q heads h0 .. h0+nh of sequence b.
__device__ void comb_task(const Params &P, const InstrAtt &I)
{
    const int b = (int)I.b;
    if (b >= P.batch) return;
    const int D = P.head_dim, nc = (int)I.nc;
    const float *part = (const float *)(P.ws + P.lay.act) + I.out;
    float *o = (float *)(P.ws + P.lay.act) + I.o_out + (size_t)b * I.o_ld;
    for (int e = threadIdx.x; e < (int)I.nh * D; e += kWgThreads) {
        int h = (int)I.h0 + e / D, i = e % D;
        const float *src = part + (((size_t)b * P.n_q_heads + h) * nc) * (D + 2);
        float M = -INFINITY;
        for (int c = 0; c < nc; ++c) M = fmaxf(M, src[(size_t)c * (D + 2) + D]);
        float L = 0.f, A = 0.f;
        for (int c = 0; c < nc; ++c) {
            const float *s = src + (size_t)c * (D + 2);
            float f = safe_exp_diff(s[D], M);
            L += s[D + 1] * f;
            A += s[i] * f;
        }
        o[(size_t)h * D + i] = A / L;
    }
}

// ---------------------------------------------------------------- interpreter
template <bool PERSISTENT>
__device__ void run_list(const Params &P, const LdsPlan lp)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const uint32_t wg = blockIdx.x;
    const uint32_t *list = (const uint32_t *)(P.ws + P.lay.instr) + (size_t)wg * P.max_instr * kInstrDwords;
    uint32_t *sinstr = (uint32_t *)(lds + kLdsInstr);
    uint32_t *sflag = (uint32_t *)(lds + kLdsMisc + 128);
    const uint32_t *counters = (const uint32_t *)(P.ws + P.lay.counters);
    uint64_t *trace = (uint64_t *)(P.ws + P.lay.trace);
    bool dead = false;   // a wait timed out: stop waiting, keep walking so the grid drains

    for (uint32_t pc = 0; pc < P.max_instr; ++pc) {
        __syncthreads();
        if (tid < kInstrDwords) sinstr[tid] = list[(size_t)pc * kInstrDwords + tid];
        __syncthreads();
        Instr I;
        {
            uint32_t *dst = (uint32_t *)&I;
#pragma unroll
            for (int j = 0; j < kInstrDwords; ++j) dst[j] = rfl(sinstr[j]);
        }
        if (I.op == OP_END) break;
        if (!PERSISTENT && I.ref_seq != P.only_seq) continue;
        uint64_t t0 = 0, t1 = 0;
        const bool tracing = PERSISTENT && (P.flags & 1u);
        if (tracing && tid == 0) t0 = wall_clock64();

        GemvStream st;
        if (I.op == OP_GEMV) gemv_issue(P, I, st);

        if (PERSISTENT) {
            if (tid == 0) {
                uint32_t ok = 1;
                if (!dead) {
#pragma unroll
                    for (int k = 0; k < 2; ++k)
                        if (ok && I.wait_ctr[k] != kNone)
                            ok = wait_counter(counters + (size_t)I.wait_ctr[k] * kCounterStride,
                                              P.epoch * I.wait_cnt[k], P.spin_limit) ? 1u : 0u;
                }
                if (!ok) set_err(P, 0, 1u + pc);
                sflag[0] = ok;
            }
            __syncthreads();
            if (sflag[0] == 0) dead = true;
        }
        if (tracing && tid == 0) t1 = wall_clock64();

        if (I.op == OP_GEMV) {
            if (I.flags & F_MFMA) {
                if (!(I.flags & F_SKIP_PRO)) gemv_prologue<true>(P, I, lds, lp, P.batch);
                gemv_main<true>(P, I, lds, lp, st, P.batch);
            } else {
                if (!(I.flags & F_SKIP_PRO)) gemv_prologue<false>(P, I, lds, lp, 1);
                gemv_main<false>(P, I, lds, lp, st, 1);
            }
        } else if (I.op == OP_ATT) {
            const InstrAtt &A = *(const InstrAtt *)&I;
            if (P.head_dim == 128) att_task<128>(P, A, lds, lp);
            else att_task<64>(P, A, lds, lp);
        } else if (I.op == OP_COMB) {
            comb_task(P, *(const InstrAtt *)&I);
        }

        if (PERSISTENT && I.sig_ctr != kNone) {
            // every wave's stores have left the wave before the barrier; thread 0 then
            // publishes them (agent-scope release) with the counter increment
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (tid == 0)
                __hip_atomic_fetch_add((uint32_t *)counters + (size_t)I.sig_ctr * kCounterStride, 1u,
                                       __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (tracing && tid == 0) {
            uint64_t *r = trace + ((size_t)wg * P.max_instr + pc) * 4;
            r[0] = ((uint64_t)wg << 32) | pc; r[1] = t0; r[2] = t1; r[3] = wall_clock64();
        }
    }
}

}  // namespace mk

extern "C" __global__ void __launch_bounds__(mk::kWgThreads)
mk_megakernel(const mk::Params P, const mk::LdsPlan lp) { mk::run_list<true>(P, lp); }

extern "C" __global__ void __launch_bounds__(mk::kWgThreads)
mk_op_kernel(const mk::Params P, const mk::LdsPlan lp) { mk::run_list<false>(P, lp); }

// Offline weight reorder: row-major bf16 [n_rows][n_cols] -> tile-major chunks.
// Destination row block of source row block rb is rb0 + rb * rb_stride (so two
// matrices can be interleaved block-wise); chunk (rb, kb) holds lane-major
// 16 B: lane = ksub * 16 + r -> 8 elements W[rb*16 + r][kb*32 + ksub*8 + 0..7].
extern "C" __global__ void mk_repack_kernel(const uint16_t *src, int n_rows, int n_cols, mk::u32x4 *dst,
                                            uint32_t kbt, uint32_t rb0, uint32_t rb_stride, uint32_t n_rb)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)n_rb * kbt * 64;
    if (gid >= total) return;
    uint32_t lane = (uint32_t)(gid & 63);
    size_t ck = gid >> 6;
    uint32_t kb = (uint32_t)(ck % kbt), rb = (uint32_t)(ck / kbt);
    int row = (int)(rb * 16 + (lane & 15));
    int k0 = (int)(kb * 32 + (lane >> 4) * 8);
    uint16_t e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int k = k0 + j;
        e[j] = (row < n_rows && k < n_cols) ? src[(size_t)row * n_cols + k] : (uint16_t)0;
    }
    mk::u32x4 v;
    v.x = e[0] | ((uint32_t)e[1] << 16); v.y = e[2] | ((uint32_t)e[3] << 16);
    v.z = e[4] | ((uint32_t)e[5] << 16); v.w = e[6] | ((uint32_t)e[7] << 16);
    dst[((size_t)(rb0 + rb * rb_stride) * kbt + kb) * 64 + lane] = v;
}

extern "C" __global__ void mk_copy_u16_kernel(const uint16_t *src, uint16_t *dst, size_t n)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < n) dst[gid] = src[gid];
}

extern "C" __global__ void mk_fill_u32_kernel(uint32_t *dst, uint32_t v, size_t n)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < n) dst[gid] = v;
}
