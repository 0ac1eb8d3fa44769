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
// that do not depend on the previous operator are issued before the dependency
// wait -- through the LDS page ring the whole weight stream of a workgroup runs
// ahead of its consumers across task boundaries; without a ring the first
// chunks of each task are loaded into registers before the wait.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "mk_isa.h"

namespace mk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct LdsPlan {
    uint32_t red_bytes;   // cross-wave reduction region
    uint32_t xs_off;      // byte offset of the staged-input region
    uint32_t ring_off;    // byte offset of the weight-page ring (1 KB aligned)
    uint32_t ring_slots;  // 1 KB pages in the ring, a quarter per wavefront (0: no ring)
};

// Per-wave view of the workgroup: LDS plan plus the state of this wavefront's weight-page ring.
//
// Page ring (persistent kernel with ring_slots > 0; paper Sec. 4.1.1 pages, Sec. 4.2.2 Step 3 page
// states, Sec. 4.2.3 decoupled weight loads).  The weight chunks a workgroup consumes over the
// whole step form one static stream (its GEMV tasks in list order); wavefront w owns the chunks
// with task-local index w, w+4, ... of every task.  Each wavefront streams its own chunks into
// its own ring of S = ring_slots / 4 pages with 128-bit global->LDS DMA loads, up to S chunks
// ahead of its consumption and across task and operator boundaries: weights depend on nothing,
// so HBM streaming continues while the workgroup waits on dependency counters.  A page is
// Locked from the DMA issue until the wavefront's in-order load counter shows it has landed,
// Ready until the wavefront has read it into registers, then refilled at once.  Pages are
// handled in stages of kStagePages: a stage holds up to four consecutive chunks of ONE task (the
// last stage of a task may be partly used), is filled by one burst of DMA loads and read back
// by one burst of LDS reads.  Because a wavefront only reads pages it filled itself, the ring
// needs no cross-wave synchronisation.  All fields are wave-uniform.
constexpr uint32_t kStagePages = 4;
typedef const __attribute__((address_space(4))) uint32_t *cptr;   // data that never changes during a launch
struct Wg {
    uint32_t red_bytes, xs_off;
    bool ring;            // weights come through the page ring (else: straight into registers)
    int npf;              // 128-bit weight loads a lane keeps in flight (direct-load path), <= kPrefetch
    uint32_t pc;          // index of the instruction being executed (task trace)
    uint32_t wave;
    uint32_t ring_off;    // byte offset of this wave's page 0 from the LDS base
    uint32_t ring_lds;    // LDS address of this wave's page 0
    uint32_t nst;         // stages (groups of kStagePages pages) of this wave
    uint32_t head, tail;  // chunks this wave has issued / read back
    uint32_t hst, tst;    // stage the next group is loaded into / read from
    cptr pf_ptr;          // next entry of the workgroup's stream table
    cptr pf_begin;        // first entry (the stream repeats once per decode step of the launch)
    uint32_t pf_steps;    // steps whose stream has not been started yet
    uint32_t pf_left;     // table entries not yet read in this pass (bounds the walk)
    const char *pf_src;   // address of this wave's next chunk in the current entry
    uint32_t pf_rem;      // chunks of the current entry this wave has not issued yet
    bool pf_live;
    // ---- the decode step this walk of the list belongs to (a launch may walk the list several times)
    uint32_t epoch;             // dependency-counter epoch of the step
    int pos_off;                // added to the caller's positions: steps done so far in this launch
    const int32_t *tok_src;     // tokens decoded by this step: the caller's, or the previous step's greedy tokens
    int32_t *tok_out;           // where this step's greedy tokens go
    float *logits;              // where this step's logits go
};

// Workgroup barrier for LDS hand-offs.  __syncthreads() would also drain every outstanding global
// access of the wave (s_waitcnt vmcnt(0)): the weight prefetch in flight, and at task boundaries the
// acknowledgement of the signal atomic -- a memory round trip per barrier that nothing here needs.
// Only LDS traffic has to be complete; global data that crosses waves is drained explicitly where
// a signal publishes it.
__device__ __forceinline__ void wg_sync(Wg &, char *)
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ uint32_t rfl(uint32_t v);
template <class T>
__device__ __forceinline__ T *rfl_ptr(T *p)
{
    const uint64_t a = (uint64_t)(uintptr_t)p;
    return (T *)(uintptr_t)((uint64_t)rfl((uint32_t)a) | ((uint64_t)rfl((uint32_t)(a >> 32)) << 32));
}
// The ring state is wave-uniform by construction.  Re-reading it through readfirstlane at every
// instruction boundary keeps it in scalar registers whatever the compiler's divergence analysis
// concludes about the surrounding control flow.
__device__ __forceinline__ void pin_uniform(Wg &wg)
{
    wg.head = rfl(wg.head); wg.tail = rfl(wg.tail); wg.hst = rfl(wg.hst); wg.tst = rfl(wg.tst);
    wg.pf_rem = rfl(wg.pf_rem); wg.pf_left = rfl(wg.pf_left); wg.pf_steps = rfl(wg.pf_steps);
    wg.pf_live = rfl((uint32_t)wg.pf_live) != 0;
    wg.pf_src = rfl_ptr(wg.pf_src);
    wg.pf_ptr = (cptr)(uintptr_t)rfl_ptr((const uint32_t *)(uintptr_t)wg.pf_ptr);
    wg.epoch = rfl(wg.epoch); wg.pos_off = (int)rfl((uint32_t)wg.pos_off);
}

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

// Activations, partial sums and counters cross workgroups (and XCDs, whose L2 caches are not
// coherent with each other) inside one launch.  They are moved with agent-scope relaxed
// atomics -- write-through stores and cache-bypassing loads (the sc1 bit) -- so that no
// L2-wide write-back / invalidate is ever needed; weights and the KV history are read-only
// during a launch and use ordinary (nontemporal) loads.
__device__ __forceinline__ float ld_act(const float *p)
{
    typedef const __attribute__((address_space(1))) uint32_t *gptr;
    return __uint_as_float(__hip_atomic_load((gptr)(uintptr_t)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void st_act(float *p, float v)
{
    typedef __attribute__((address_space(1))) uint32_t *gptr;
    __hip_atomic_store((gptr)(uintptr_t)p, __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Cross-lane sums inside a 16-lane row with DPP (no LDS crossbar traffic).  Every step pairs
// lanes symmetrically, so all lanes of the group end with bit-identical sums.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row_sum8(float v)    // over aligned groups of 8 lanes
{
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);   // row_half_mirror
    return v;
}
__device__ __forceinline__ float row_sum16(float v)   // over a 16-lane row
{
    v = row_sum8(v);
    v = dpp_add<0x140>(v);   // row_mirror
    return v;
}

template <int CTRL>
__device__ __forceinline__ float dpp_max(float v)
{
    return fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true)));
}
__device__ __forceinline__ float row_max16(float v)   // over a 16-lane row (all 16 lanes active)
{
    v = dpp_max<0xB1>(v);
    v = dpp_max<0x4E>(v);
    v = dpp_max<0x141>(v);
    v = dpp_max<0x140>(v);
    return v;
}

// Whole-wavefront reductions without LDS-crossbar shuffles (all 64 lanes active): the 16-lane rows
// first, then the row totals travel down the wave with the two row-broadcast DPP steps (lane 15 of
// a row into the next row, lane 31 into the upper half); the last lane's value goes to every lane.
__device__ __forceinline__ float wave_sum(float v)
{
    v = row_sum16(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x142, 0xa, 0xf, false));   // row_bcast:15
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x143, 0xc, 0xf, false));   // row_bcast:31
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v)
{
    v = row_max16(v);
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), 0x142, 0xa, 0xf, false)));
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), 0x143, 0xc, 0xf, false)));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ void set_err(const Params &P, int slot, uint32_t v)
{
    uint32_t *e = (uint32_t *)(P.scr + P.lay.err);
    __hip_atomic_store(e + slot, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A dependency counter is kept as kCounterSubs sub-counters on separate 128-byte lines: a producer adds to
// the one picked by its workgroup id, so the read-modify-writes of a level with hundreds of producers
// spread over that many lines instead of queueing on one.  The count is the sum of the sub-counters
// (each only grows, so a sum of reads taken at different times can only under-count).
__device__ __forceinline__ const uint32_t *sub_counter(const Params &P, const uint32_t *counters, uint32_t idx, uint32_t j)
{
    (void)P;
    return counters + ((size_t)idx * kCounterSubs + j) * kCounterStride;
}

// Wave-wide poll of a dependency counter until it has received `target` signals (wrap-safe); lane j
// reads sub-counter j.  Bounded: after `limit` polls the wait gives up and reports failure, so every
// wave always reaches the end of its instruction list.  All 64 lanes call it and get the same result.
__device__ __forceinline__ bool wait_counter(const Params &P, const uint32_t *counters, uint32_t idx, uint32_t target,
                                             uint32_t *polls = nullptr)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t *mine = sub_counter(P, counters, idx, lane & (kCounterSubs - 1u));
    uint32_t it = 0;
    bool ok = true;
    for (;;) {
        uint32_t v = lane < (uint32_t)kCounterSubs ? __hip_atomic_load(mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
        // sum over the first 32 lanes: DPP inside the 16-lane rows (integer adds), one cross-row step
        v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);    // quad_perm [1,0,3,2]
        v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true);    // quad_perm [2,3,0,1]
        v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, true);   // row_half_mirror
        v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, true);   // row_mirror
        v = rfl(v);
        if ((int32_t)(v - target) >= 0) break;
        if (++it > P.spin_limit) { ok = false; break; }
    }
    if (polls) *polls += it + 1;
    return ok;
}

__device__ __forceinline__ int clamp_i(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// Tokens may have been written by another workgroup earlier in the same launch (greedy feedback):
// read them past the caches, like every other cross-workgroup value.
__device__ __forceinline__ int token_of(const Params &P, const Wg &wg, int b)
{
    typedef const __attribute__((address_space(1))) uint32_t *gptr;
    int t = (int)rfl(__hip_atomic_load((gptr)(uintptr_t)(wg.tok_src + b), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    if (t < 0 || t >= P.vocab) { set_err(P, 1, 1u); t = clamp_i(t, 0, P.vocab - 1); }
    return t;
}
__device__ __forceinline__ int position_of(const Params &P, const Wg &wg, int b)
{
    int p = (int)rfl((uint32_t)P.positions[b]) + wg.pos_off;
    if (p < 0 || p >= P.max_context) { set_err(P, 1, 2u); p = clamp_i(p, 0, P.max_context - 1); }
    return p;
}

// Element (row, k) of a tile-major matrix whose first chunk is `chunk0` (R = 1 << rlog rows per chunk).
__device__ __forceinline__ float tile_elem(const char *wbase, uint32_t chunk0, uint32_t kbt, uint32_t rlog, int row, int k)
{
    const uint32_t R = 1u << rlog, ck = chunk_k(rlog);
    size_t chunk = (size_t)chunk0 + (size_t)((uint32_t)row >> rlog) * kbt + (size_t)((uint32_t)k / ck);
    uint32_t slot = (((uint32_t)k % ck) >> 3) * R + ((uint32_t)row & (R - 1));
    const uint16_t *p = (const uint16_t *)(wbase + chunk * kChunkBytes + slot * 16) + (k & 7);
    return bf_to_f(*p);
}

// 128-bit cache-bypassing (sc1) accesses to the activation region through a buffer descriptor;
// the compiler tracks their completion, so several can be in flight per lane.
struct ActBuf {
    __amdgpu_buffer_rsrc_t r;
};
__device__ __forceinline__ ActBuf act_buf(const Params &P)
{
    ActBuf a;
    a.r = __builtin_amdgcn_make_buffer_rsrc((void *)(P.scr + P.lay.act), 0, (int)P.act_bytes, 0x00020000);
    return a;
}
constexpr int kAuxSc1 = 16;
__device__ __forceinline__ f32x4 ld_act4(const ActBuf &a, uint32_t float_off)
{
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(a.r, (int)(float_off * 4u), 0, kAuxSc1));
}
__device__ __forceinline__ void st_act4(const ActBuf &a, uint32_t float_off, f32x4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), a.r, (int)(float_off * 4u), 0, kAuxSc1);
}

// byte N of a dword as a float (selected as v_cvt_f32_ubyteN)
template <int N>
__device__ __forceinline__ float ubyte_f(uint32_t v) { return (float)((v >> (8 * N)) & 0xffu); }

// (value, index) maximum over a wavefront; equal values keep the smaller index.  All lanes end with the result.
__device__ __forceinline__ void argmax_wave(float &v, uint32_t &i)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const float ov = __shfl_xor(v, o, 64);
        const uint32_t oi = (uint32_t)__shfl_xor((int)i, o, 64);
        if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
    }
}

// ---------------------------------------------------------------- GEMV task
// Staged input in LDS:
//   VALU path (batch 1): fp32 x[k]
//   MFMA path: bf16 planes [col][k], col = b * nterm + term, x = sum of its nterm bf16 terms;
//              plane stride = k_stage * 2 + 16 bytes (bank skew)
// Two fp32 values to a packed pair of bf16 (round to nearest even) with the hardware conversion
// (v_cvt_pk_bf16_f32).  Used for the activation split only: the KV rows are rounded by f_to_bf,
// whose integer arithmetic is the same on every input as the oracle's.
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

template <bool MFMA>
__device__ __forceinline__ void store_x4(char *xs, int b, int i, f32x4 y, int nterm, uint32_t plane_stride)
{
    if (!MFMA) {
        *(f32x4 *)(xs + (size_t)i * 4) = y;
    } else {
        f32x4 r = y;
        for (int t = 0; t < nterm; ++t) {
            uint2 pk;
            pk.x = pack_bf16x2(r.x, r.y);
            pk.y = pack_bf16x2(r.z, r.w);
            *(uint2 *)(xs + (size_t)(b * nterm + t) * plane_stride + (size_t)i * 2) = pk;
            r.x -= bf_lo(pk.x); r.y -= bf_hi(pk.x); r.z -= bf_lo(pk.y); r.w -= bf_hi(pk.y);
        }
    }
}

// bf16 terms an fp32 activation is split into on the matrix-core path: hi + lo keeps 16 mantissa
// bits (relative error 2^-17 per activation, far inside the tolerance), and up to 8 sequences x 2
// terms fill the 16 columns of the instruction.  A third term measured 7 % slower at batch 4.
__device__ __forceinline__ int nterm_of(int) { return kActTerms; }

constexpr int kQuadsPerThread = 4;   // hidden <= 4 * 4 * 256

// Matrix-core path, several sequences: the same staging as gemv_prologue, organised so that the loads
// of ALL sequences are in flight together.  A lane walks the flattened (sequence, quad) items in
// groups of kItems; one memory round trip then covers kItems quads per lane instead of one sequence.
// The normalising forms park the summed rows as fp32 inside each sequence's own (larger) plane region,
// take the sum of squares with one wave per sequence, and rewrite the region as bf16 planes.
// Returns false for the forms it does not cover (the caller's per-sequence code handles those).
constexpr int kItems = 8;

__device__ __forceinline__ bool gemv_prologue_batched(const Params &P, const Instr &I, char *lds, Wg &lp, int batch)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = (int)rfl((uint32_t)tid >> 6);
    char *xs = lds + lp.xs_off;
    float *misc = (float *)(lds + kLdsMisc);
    const ActBuf ab = act_buf(P);
    const int nterm = nterm_of(P.max_batch);
    const uint32_t pro = instr_pro(I), n_parts = instr_nparts(I);
    constexpr uint32_t kNone = 0xfffffff0u;            // beyond the descriptor: the load returns zeros

    if (pro == PRO_EMBED_NORM || pro == PRO_RESID_NORM) {
        const int H = P.hidden, nq4 = H >> 2, total = batch * nq4;
        const uint32_t plane_stride = (uint32_t)H * 2u + 16u, seq_stride = (uint32_t)nterm * plane_stride;
        const uint16_t *gain = (const uint16_t *)(P.ws + P.lay.vecs) + I.gain;
        uint2 gw[kQuadsPerThread];                       // constants: fetched with the input loads
#pragma unroll
        for (int j = 0; j < kQuadsPerThread; ++j) {
            const int q = tid + j * kWgThreads;
            gw[j] = q < nq4 ? *(const uint2 *)(gain + 4 * q) : uint2{0u, 0u};
        }
        for (int e0 = tid; e0 < total; e0 += kWgThreads * kItems) {
            f32x4 v[kItems];
            uint32_t off[kItems];                        // b * in_ld + 4 q of the item, kNone past the end
            int bq[kItems];                              // b << 16 | q
#pragma unroll
            for (int u = 0; u < kItems; ++u) {
                const int e = e0 + u * kWgThreads;
                const int b = e / nq4, q = e - b * nq4;
                off[u] = e < total ? (uint32_t)b * I.in_ld + 4u * (uint32_t)q : kNone;
                bq[u] = (b << 16) | q;
            }
            if (pro == PRO_EMBED_NORM) {
#pragma unroll
                for (int u = 0; u < kItems; ++u) {
                    f32x4 x = {0.f, 0.f, 0.f, 0.f};
                    if (off[u] != kNone) {
                        const int tok = token_of(P, lp, bq[u] >> 16), k = 4 * (bq[u] & 0xffff);
                        x.x = tile_elem(P.ws + P.lay.weights, P.embed_chunk, P.embed_kbt, P.embed_rlog, tok, k);
                        x.y = tile_elem(P.ws + P.lay.weights, P.embed_chunk, P.embed_kbt, P.embed_rlog, tok, k + 1);
                        x.z = tile_elem(P.ws + P.lay.weights, P.embed_chunk, P.embed_kbt, P.embed_rlog, tok, k + 2);
                        x.w = tile_elem(P.ws + P.lay.weights, P.embed_chunk, P.embed_kbt, P.embed_rlog, tok, k + 3);
                    }
                    v[u] = x;
                }
            } else {
#pragma unroll
                for (int u = 0; u < kItems; ++u) v[u] = ld_act4(ab, off[u] != kNone ? I.in_base + off[u] : kNone);
                // the producer's partial sums, two partials of every item in flight, added in order
                for (uint32_t s0 = 0; s0 < n_parts; s0 += 2) {
                    f32x4 t0[kItems], t1[kItems];
                    const uint32_t p0 = I.in_parts + s0 * I.part_stride, p1 = p0 + I.part_stride;
                    const bool two = s0 + 1 < n_parts;
#pragma unroll
                    for (int u = 0; u < kItems; ++u) {
                        t0[u] = ld_act4(ab, off[u] != kNone ? p0 + off[u] : kNone);
                        t1[u] = ld_act4(ab, (two && off[u] != kNone) ? p1 + off[u] : kNone);
                    }
#pragma unroll
                    for (int u = 0; u < kItems; ++u) { v[u] += t0[u]; v[u] += t1[u]; }
                }
            }
#pragma unroll
            for (int u = 0; u < kItems; ++u) {
                if (off[u] == kNone) continue;
                const int b = bq[u] >> 16, q = bq[u] & 0xffff;
                if ((uint32_t)(4 * q) >= I.xs_lo && (uint32_t)(4 * q) < I.xs_hi) st_act4(ab, I.xs_out + off[u], v[u]);
                *(f32x4 *)(xs + (size_t)b * seq_stride + (size_t)q * 16) = v[u];
            }
        }
        wg_sync(lp, lds);
        // The planes of a sequence overwrite its parked row.  Every lane takes its part of the rows of up to kSeqGroup
        // sequences into registers and adds up its squares (summed over the wavefront with DPP, the four wavefront sums
        // meet in LDS); one barrier later the rows are scaled and written as planes -- one LDS round trip and one barrier per
        // group of sequences.  The wavefront sums of consecutive groups use alternating halves of a 32-float area.
        constexpr int kSeqGroup = 4;
        for (int b0 = 0, grp = 0; b0 < batch; b0 += kSeqGroup, ++grp) {
            f32x4 v[kSeqGroup][kQuadsPerThread];
            float *part = misc + 16 * (grp & 1);
#pragma unroll
            for (int g = 0; g < kSeqGroup; ++g) {
                const f32x4 *vp = (const f32x4 *)(xs + (size_t)min(b0 + g, batch - 1) * seq_stride);
                float ss = 0.f;
#pragma unroll
                for (int j = 0; j < kQuadsPerThread; ++j) {
                    const int q = tid + j * kWgThreads;
                    v[g][j] = q < nq4 ? vp[q] : f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int j = 0; j < kQuadsPerThread; ++j)
                    ss += (v[g][j].x * v[g][j].x + v[g][j].y * v[g][j].y) + (v[g][j].z * v[g][j].z + v[g][j].w * v[g][j].w);
                ss = wave_sum(ss);
                if (lane == 0) part[g * kWaves + wave] = ss;
            }
            wg_sync(lp, lds);
#pragma unroll
            for (int g = 0; g < kSeqGroup; ++g) {
                const int b = b0 + g;
                if (b >= batch) break;
                const float tot = (part[g * kWaves] + part[g * kWaves + 1]) + (part[g * kWaves + 2] + part[g * kWaves + 3]);
                const float inv = 1.0f / sqrtf(tot / (float)H + P.rms_eps);
#pragma unroll
                for (int j = 0; j < kQuadsPerThread; ++j) {
                    const int q = tid + j * kWgThreads;
                    if (q < nq4) {
                        f32x4 y;
                        y.x = v[g][j].x * inv * bf_lo(gw[j].x); y.y = v[g][j].y * inv * bf_hi(gw[j].x);
                        y.z = v[g][j].z * inv * bf_lo(gw[j].y); y.w = v[g][j].w * inv * bf_hi(gw[j].y);
                        store_x4<true>(xs, b, 4 * q, y, nterm, plane_stride);
                    }
                }
            }
        }
        return true;
    }

    const bool plain1 = pro == PRO_PLAIN && n_parts == 1;
    if (!plain1 && pro != PRO_SILU) return false;
    const uint32_t ck = instr_ck(I);
    const int k0 = (int)(I.xs_lo * ck), kn = (int)(I.xs_hi * ck), nq = kn >> 2, total = batch * nq;
    const uint32_t plane_stride = (uint32_t)kn * 2u + 16u;
    if (plain1) {
        for (int e0 = tid; e0 < total; e0 += kWgThreads * kItems) {
            f32x4 y[kItems];
#pragma unroll
            for (int u = 0; u < kItems; ++u) {
                const int e = e0 + u * kWgThreads;
                const int b = e / nq, i = 4 * (e - b * nq);
                const uint32_t k = (uint32_t)(k0 + i);
                y[u] = ld_act4(ab, (e < total && k < I.k_len) ? I.in_parts + (uint32_t)b * I.in_ld + k : kNone);
            }
#pragma unroll
            for (int u = 0; u < kItems; ++u) {
                const int e = e0 + u * kWgThreads;
                const int b = e / nq, i = 4 * (e - b * nq);
                const uint32_t k = (uint32_t)(k0 + i);
                if (k + 1 >= I.k_len) y[u].y = 0.f;      // elements at or beyond the true K are zero
                if (k + 2 >= I.k_len) y[u].z = 0.f;
                if (k + 3 >= I.k_len) y[u].w = 0.f;
                if (e < total) store_x4<true>(xs, b, i, y[u], nterm, plane_stride);
            }
        }
        return true;
    }
    // SILU over the fused gate/up output: row group j holds PR/2 gate rows then PR/2 up rows (PR >= 8)
    constexpr int kIt = kItems / 2;                      // gate and up of two partials: 4 loads per item in flight
    const uint32_t PR = 1u << instr_prod_rlog(I), half = PR >> 1;
    for (int e0 = tid; e0 < total; e0 += kWgThreads * kIt) {
        f32x4 gs[kIt], us[kIt];
        uint32_t src[kIt];
#pragma unroll
        for (int u = 0; u < kIt; ++u) {
            const int e = e0 + u * kWgThreads;
            const int b = e / nq, i = 4 * (e - b * nq);
            const uint32_t k = (uint32_t)(k0 + i);
            src[u] = (e < total && k < I.k_len) ? (uint32_t)b * I.in_ld + (k / half) * PR + (k % half) : kNone;
            gs[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            us[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        for (uint32_t s0 = 0; s0 < n_parts; s0 += 2) {
            f32x4 g0[kIt], u0[kIt], g1[kIt], u1[kIt];
            const uint32_t p0 = I.in_parts + s0 * I.part_stride, p1 = p0 + I.part_stride;
            const bool two = s0 + 1 < n_parts;
#pragma unroll
            for (int u = 0; u < kIt; ++u) {
                const bool ok = src[u] != kNone;
                g0[u] = ld_act4(ab, ok ? p0 + src[u] : kNone);
                u0[u] = ld_act4(ab, ok ? p0 + src[u] + half : kNone);
                g1[u] = ld_act4(ab, (ok && two) ? p1 + src[u] : kNone);
                u1[u] = ld_act4(ab, (ok && two) ? p1 + src[u] + half : kNone);
            }
#pragma unroll
            for (int u = 0; u < kIt; ++u) { gs[u] += g0[u]; us[u] += u0[u]; gs[u] += g1[u]; us[u] += u1[u]; }
        }
#pragma unroll
        for (int u = 0; u < kIt; ++u) {
            const int e = e0 + u * kWgThreads;
            const int b = e / nq, i = 4 * (e - b * nq);
            const uint32_t k = (uint32_t)(k0 + i);
            f32x4 acc;
            acc.x = gs[u].x / (1.0f + __expf(-gs[u].x)) * us[u].x; acc.y = gs[u].y / (1.0f + __expf(-gs[u].y)) * us[u].y;
            acc.z = gs[u].z / (1.0f + __expf(-gs[u].z)) * us[u].z; acc.w = gs[u].w / (1.0f + __expf(-gs[u].w)) * us[u].w;
            if (k + 1 >= I.k_len) acc.y = 0.f;
            if (k + 2 >= I.k_len) acc.z = 0.f;
            if (k + 3 >= I.k_len) acc.w = 0.f;
            if (e < total) store_x4<true>(xs, b, i, acc, nterm, plane_stride);
        }
    }
    return true;
}

template <bool MFMA>
__device__ __forceinline__ void gemv_prologue(const Params &P, const Instr &I, char *lds, Wg &lp, int batch)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = (int)rfl((uint32_t)tid >> 6);
    char *xs = lds + lp.xs_off;
    float *misc = (float *)(lds + kLdsMisc);
    const ActBuf ab = act_buf(P);
    const int nterm = nterm_of(P.max_batch);
    const uint32_t pro = instr_pro(I), n_parts = instr_nparts(I);

    // Matrix-core W4 tasks: behind the planes, per plane, the sums of every 32 consecutive staged bf16 values (the
    // zero point of a group of codes is 136 times the sum of the group's staged values: codes enter the matrix cores
    // as the bf16 numbers 128 + q).  Summed from the rounded plane values, so that it cancels exactly what the
    // products carry.
    auto plane_sums = [&]() {
        if (!(MFMA && (I.flags & F_W4))) return;
        const bool nk = (pro == PRO_EMBED_NORM || pro == PRO_RESID_NORM);
        const uint32_t ks = nk ? (uint32_t)P.hidden : I.xs_hi * instr_ck(I);
        const uint32_t pstride = ks * 2u + 16u, nblk = ks / 32u, ncol = (uint32_t)(batch * nterm);
        float *xsum = (float *)(xs + (size_t)(P.max_batch * nterm) * pstride);
        for (uint32_t e = tid; e < ncol * nblk; e += kWgThreads) {
            const uint32_t col = e / nblk, blk = e - col * nblk;
            const u32x4 *xp = (const u32x4 *)(xs + (size_t)col * pstride + (size_t)blk * 64);
            u32x4 xv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) xv[i] = xp[i];
            float a = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a += bf_lo(xv[i].x); a += bf_hi(xv[i].x); a += bf_lo(xv[i].y); a += bf_hi(xv[i].y);
                a += bf_lo(xv[i].z); a += bf_hi(xv[i].z); a += bf_lo(xv[i].w); a += bf_hi(xv[i].w);
            }
            xsum[e] = a;
        }
        wg_sync(lp, lds);
    };
    if constexpr (MFMA) {
        if (batch > 1 && gemv_prologue_batched(P, I, lds, lp, batch)) {
            wg_sync(lp, lds);
            plane_sums();
            return;
        }
    }
    if (pro == PRO_EMBED_NORM || pro == PRO_RESID_NORM) {
        const int H = P.hidden, nq4 = H >> 2;
        const uint32_t plane_stride = (uint32_t)H * 2u + 16u;
        const uint16_t *gain = (const uint16_t *)(P.ws + P.lay.vecs) + I.gain;
        // the gains are constants: fetch them first, so that they travel with the input loads
        uint2 gw[kQuadsPerThread];
#pragma unroll
        for (int j = 0; j < kQuadsPerThread; ++j) {
            const int q = tid + j * kWgThreads;
            gw[j] = q < nq4 ? *(const uint2 *)(gain + 4 * q) : uint2{0u, 0u};
        }
        for (int b = 0; b < batch; ++b) {
            f32x4 v[kQuadsPerThread];
            if (pro == PRO_EMBED_NORM) {
                const int tok = token_of(P, lp, b);
#pragma unroll
                for (int j = 0; j < kQuadsPerThread; ++j) {
                    const int q = tid + j * kWgThreads;
                    f32x4 x = {0.f, 0.f, 0.f, 0.f};
                    if (q < nq4) {
                        x.x = tile_elem(P.ws + P.lay.weights, P.embed_chunk, P.embed_kbt, P.embed_rlog, tok, 4 * q);
                        x.y = tile_elem(P.ws + P.lay.weights, P.embed_chunk, P.embed_kbt, P.embed_rlog, tok, 4 * q + 1);
                        x.z = tile_elem(P.ws + P.lay.weights, P.embed_chunk, P.embed_kbt, P.embed_rlog, tok, 4 * q + 2);
                        x.w = tile_elem(P.ws + P.lay.weights, P.embed_chunk, P.embed_kbt, P.embed_rlog, tok, 4 * q + 3);
                    }
                    v[j] = x;
                }
            } else {
                const uint32_t row = I.in_base + (uint32_t)b * I.in_ld;
#pragma unroll
                for (int j = 0; j < kQuadsPerThread; ++j) {
                    const int q = tid + j * kWgThreads;
                    v[j] = ld_act4(ab, q < nq4 ? row + 4u * q : 0xfffffff0u);   // out of range reads return 0
                }
                // partial sums of the producer, four partials (x four quads) in flight at a time, added in order
                for (uint32_t s0 = 0; s0 < n_parts; s0 += 4) {
                    f32x4 t[4][kQuadsPerThread];
#pragma unroll
                    for (int ds = 0; ds < 4; ++ds) {
                        const uint32_t prow = I.in_parts + (s0 + ds) * I.part_stride + (uint32_t)b * I.in_ld;
#pragma unroll
                        for (int j = 0; j < kQuadsPerThread; ++j) {
                            const int q = tid + j * kWgThreads;
                            t[ds][j] = ld_act4(ab, (q < nq4 && s0 + ds < n_parts) ? prow + 4u * q : 0xfffffff0u);
                        }
                    }
#pragma unroll
                    for (int ds = 0; ds < 4; ++ds)
#pragma unroll
                        for (int j = 0; j < kQuadsPerThread; ++j) v[j] += t[ds][j];
                }
            }
            float ss = 0.f;
#pragma unroll
            for (int j = 0; j < kQuadsPerThread; ++j) {
                const int q = tid + j * kWgThreads;
                if (q < nq4 && (uint32_t)(4 * q) >= I.xs_lo && (uint32_t)(4 * q) < I.xs_hi)
                    st_act4(ab, I.xs_out + (uint32_t)b * I.in_ld + 4u * q, v[j]);
                ss += v[j].x * v[j].x + v[j].y * v[j].y + v[j].z * v[j].z + v[j].w * v[j].w;
            }
            ss = wave_sum(ss);
            float *slot = misc + (b & 1) * 8;
            if (lane == 0) slot[wave] = ss;
            wg_sync(lp, lds);
            float tot = slot[0] + slot[1] + slot[2] + slot[3];
            float inv = 1.0f / sqrtf(tot / (float)H + P.rms_eps);
#pragma unroll
            for (int j = 0; j < kQuadsPerThread; ++j) {
                const int q = tid + j * kWgThreads;
                if (q < nq4) {
                    f32x4 y;
                    y.x = v[j].x * inv * bf_lo(gw[j].x); y.y = v[j].y * inv * bf_hi(gw[j].x);
                    y.z = v[j].z * inv * bf_lo(gw[j].y); y.w = v[j].w * inv * bf_hi(gw[j].y);
                    store_x4<MFMA>(xs, b, 4 * q, y, nterm, plane_stride);
                }
            }
        }
    } else {
        // PLAIN / SILU: stage chunks [xs_lo, xs_lo + xs_hi) of the input (whole-K chunk indices)
        const uint32_t ck = instr_ck(I);
        const int k0 = (int)(I.xs_lo * ck), kn = (int)(I.xs_hi * ck);
        const uint32_t plane_stride = (uint32_t)kn * 2u + 16u;
        const uint32_t prl = instr_prod_rlog(I), PR = 1u << prl;
        for (int b = 0; b < batch; ++b) {
            const uint32_t brow = (uint32_t)b * I.in_ld;
            if (pro == PRO_COMBINE) {
                // The attention partials of the heads that cover this task's k range, combined here
                // (flash-decode merge in fixed chunk order) instead of by separate combine tasks.
                const int D = P.head_dim, RS = D + 4, nc = (int)n_parts;      // rows are [acc[D], m, l, pad, pad]
                const int k1 = min(k0 + kn, (int)I.k_len);
                const int h0 = k0 / D, nh = (k1 - k0) / D;
                float *stg = (float *)(xs + I.in_base);                      // [nh][nc][RS] partial rows
                float *wgt = stg + (size_t)nh * nc * RS;                     // [nh][nc] merge weights f_c / L
                const uint32_t src = I.in_parts + (uint32_t)(((size_t)b * P.n_q_heads + h0) * nc) * (uint32_t)RS;
                const int nq4 = nh * nc * RS / 4;
                if (b) wg_sync(lp, lds);                                      // the previous sequence is done with the staging
                for (int q0 = tid; q0 < nq4; q0 += kWgThreads * 4) {
                    f32x4 v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int q = q0 + u * kWgThreads;
                        v[u] = ld_act4(ab, q < nq4 ? src + 4u * q : 0xfffffff0u);
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int q = q0 + u * kWgThreads;
                        if (q < nq4) *(f32x4 *)(stg + 4 * q) = v[u];
                    }
                }
                wg_sync(lp, lds);
                for (int h = wave; h < nh; h += kWaves) {                    // one wave per head, one lane per chunk
                    const float *row = stg + ((size_t)h * nc + min(lane, nc - 1)) * RS;
                    const float m = lane < nc ? row[D] : -INFINITY, l = lane < nc ? row[D + 1] : 0.f;
                    const float M = wave_max(m);
                    const float f = (m == -INFINITY) ? 0.f : __expf(m - M);
                    const float L = wave_sum(f * l);
                    if (lane < nc) wgt[h * nc + lane] = f / L;
                }
                wg_sync(lp, lds);
                for (int q = tid; q < nh * D / 4; q += kWgThreads) {
                    const int h = (4 * q) / D, i = (4 * q) % D;
                    const float *rows = stg + (size_t)h * nc * RS + i;
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                    for (int c = 0; c < nc; ++c) acc += wgt[h * nc + c] * *(const f32x4 *)(rows + (size_t)c * RS);
                    store_x4<MFMA>(xs, b, 4 * q, acc, nterm, plane_stride);
                }
                for (int q = nh * D / 4 + tid; q < kn / 4; q += kWgThreads)   // staged k beyond the true K are zero
                    store_x4<MFMA>(xs, b, 4 * q, f32x4{0.f, 0.f, 0.f, 0.f}, nterm, plane_stride);
                continue;
            }
            if (pro == PRO_PLAIN && n_parts == 1) {
                // common case (unsplit producer): nine 128-bit loads in flight per lane, one memory round
                // trip for up to 9216 staged elements (the 8960-wide MLP of the 1.5B shape fits)
                constexpr int U = 9;
                for (int i0 = tid * 4; i0 < kn; i0 += kWgThreads * 4 * U) {
                    f32x4 y[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int i = i0 + u * kWgThreads * 4;
                        const uint32_t k = (uint32_t)(k0 + i);
                        y[u] = ld_act4(ab, (i < kn && k < I.k_len) ? I.in_parts + brow + k : 0xfffffff0u);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int i = i0 + u * kWgThreads * 4;
                        const uint32_t k = (uint32_t)(k0 + i);
                        if (k + 1 >= I.k_len) y[u].y = 0.f;
                        if (k + 2 >= I.k_len) y[u].z = 0.f;
                        if (k + 3 >= I.k_len) y[u].w = 0.f;
                        if (i < kn) store_x4<MFMA>(xs, b, i, y[u], nterm, plane_stride);
                    }
                }
                continue;
            }
            for (int i0 = tid * 4; i0 < kn; i0 += kWgThreads * 4 * 2) {
                // two quads per thread and iteration keep several loads in flight
                f32x4 y[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int i = i0 + u * kWgThreads * 4;
                    const uint32_t k = (uint32_t)(k0 + i);
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                    if (i < kn && k < I.k_len) {
                        if (pro == PRO_PLAIN) {
                            for (uint32_t s = 0; s < n_parts; ++s) acc += ld_act4(ab, I.in_parts + s * I.part_stride + brow + k);
                        } else {
                            // fused gate/up output: row group j holds PR/2 gate rows then PR/2 up rows (PR >= 8)
                            const uint32_t half = PR >> 1;
                            const uint32_t gi = (k / half) * PR + (k % half);
                            f32x4 gs = {0.f, 0.f, 0.f, 0.f}, us = {0.f, 0.f, 0.f, 0.f};
                            for (uint32_t s = 0; s < n_parts; ++s) {
                                gs += ld_act4(ab, I.in_parts + s * I.part_stride + brow + gi);
                                us += ld_act4(ab, I.in_parts + s * I.part_stride + brow + gi + half);
                            }
                            acc.x = gs.x / (1.0f + __expf(-gs.x)) * us.x; acc.y = gs.y / (1.0f + __expf(-gs.y)) * us.y;
                            acc.z = gs.z / (1.0f + __expf(-gs.z)) * us.z; acc.w = gs.w / (1.0f + __expf(-gs.w)) * us.w;
                        }
                        // elements at or beyond the true K are zero
                        if (k + 1 >= I.k_len) acc.y = 0.f;
                        if (k + 2 >= I.k_len) acc.z = 0.f;
                        if (k + 3 >= I.k_len) acc.w = 0.f;
                    }
                    y[u] = acc;
                }
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int i = i0 + u * kWgThreads * 4;
                    if (i < kn) store_x4<MFMA>(xs, b, i, y[u], nterm, plane_stride);
                }
            }
        }
    }
    wg_sync(lp, lds);
    plane_sums();
    if (!MFMA && (I.flags & F_W4)) {
        // W4: sums of every 32 consecutive staged values, behind the vector (the zero-point term of a
        // lane's 32 codes is 8 times such a sum)
        const bool nk = (pro == PRO_EMBED_NORM || pro == PRO_RESID_NORM);
        const uint32_t ks = nk ? (uint32_t)P.hidden : I.xs_hi * instr_ck(I);
        float *xsum = (float *)(xs + (size_t)ks * 4);
        for (uint32_t blk = tid; blk < ks / 32u; blk += kWgThreads) {
            const f32x4 *xp = (const f32x4 *)(xs + (size_t)blk * 128);
            f32x4 xv[8];                                   // the eight reads in flight, then the sum in order
#pragma unroll
            for (int i = 0; i < 8; ++i) xv[i] = xp[i];
            f32x4 acc = xv[0];
#pragma unroll
            for (int i = 1; i < 8; ++i) acc += xv[i];
            xsum[blk] = (acc.x + acc.y) + (acc.z + acc.w);
        }
        wg_sync(lp, lds);
    }
}

// Cursor over the units of a GEMV task in list order: (row group, K slice) of the current unit.
struct UnitCursor {
    uint32_t rg, s;
    __device__ __forceinline__ void next(bool sm, uint32_t S, uint32_t groups)
    {
        if (sm) { if (++rg == groups) { rg = 0; ++s; } }
        else    { if (++s == S) { s = 0; ++rg; } }
    }
};

// ---- weight-page ring ------------------------------------------------------------------------
// Wait until at most 4 * k4 vector-memory operations of this wave are outstanding (k4 is clamped
// to 15; rounding the allowance down only waits longer).  s_waitcnt takes its count as an
// immediate, so the wait is one entry of a table of (s_waitcnt, s_branch) pairs of 8 bytes each,
// entered through a computed jump: the three instructions between s_getpc_b64 and the table are
// 4 bytes each, hence the offset 12.
__device__ __forceinline__ void vm_wait4(uint32_t k4)
{
    uint32_t tmp;
    asm volatile(
        "s_min_u32 %0, %1, 15\n\t"
        "s_lshl_b32 %0, %0, 3\n\t"
        "s_add_u32 %0, %0, 12\n\t"
        "s_getpc_b64 vcc\n\t"
        "s_add_u32 vcc_lo, vcc_lo, %0\n\t"
        "s_addc_u32 vcc_hi, vcc_hi, 0\n\t"
        "s_setpc_b64 vcc\n\t"
        "s_waitcnt vmcnt(0)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(4)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(8)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(12)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(16)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(20)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(24)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(28)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(32)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(36)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(40)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(44)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(48)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(52)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(56)\n\ts_branch .Lvmw_%=\n\t"
        "s_waitcnt vmcnt(60)\n\ts_branch .Lvmw_%=\n"
        ".Lvmw_%=:"
        : "=&s"(tmp) : "s"(rfl(k4)) : "memory", "vcc", "scc");
}

// One 128-bit global->LDS DMA load of a 1 KB chunk: lane l's 16 bytes land at dst + 16 l.  Written
// as inline assembly on purpose: the compiler does not track it, so it never serialises the
// wave's LDS reads against the DMA queue; the ring code waits for landing itself (vm_wait4).
__device__ __forceinline__ void dma_chunk(uint32_t dst_lds, const char *src, uint32_t lane_off)
{
    // the operands are wave-uniform by construction; readfirstlane pins them to scalar registers
    const uint64_t a = (uint64_t)(uintptr_t)src;
    const uint64_t src_s = (uint64_t)rfl((uint32_t)a) | ((uint64_t)rfl((uint32_t)(a >> 32)) << 32);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 ::"s"(rfl(dst_lds)), "v"(lane_off), "s"(src_s) : "memory", "m0");
}

// Move the stream cursor to the next table entry that holds chunks of this wave (rare path).
__device__ __forceinline__ void ring_advance(const Params &P, Wg &wg)
{
    while (wg.pf_live && wg.pf_rem == 0) {
        const uint32_t base = wg.pf_left ? wg.pf_ptr[0] : kNone, total = wg.pf_left ? wg.pf_ptr[1] : kNone;
        if (total == kNone) {   // end of the step's stream: start over for the next step, if any
            if (wg.pf_steps == 0) { wg.pf_live = false; break; }
            --wg.pf_steps;
            wg.pf_ptr = wg.pf_begin; wg.pf_left = P.max_instr;
            continue;
        }
        wg.pf_ptr += 2; --wg.pf_left;
        if (total > wg.wave) {
            wg.pf_rem = (total - wg.wave + kWaves - 1) / kWaves;
            wg.pf_src = P.ws + P.lay.weights + ((size_t)base + wg.wave) * kChunkBytes;
        }
    }
}

// Fill the next stage with the next group of this wave's stream: up to four chunks of one task
// (no-op once the stream is exhausted).  Consecutive chunks of a wave are kWaves chunks apart.
__device__ __forceinline__ void ring_fill_stage(const Params &P, Wg &wg)
{
    if (wg.pf_rem == 0) ring_advance(P, wg);
    if (!wg.pf_live) return;
    const uint32_t lane_off = (threadIdx.x & 63u) * 16u;
    const uint32_t dst = wg.ring_lds + wg.hst * (kStagePages * kChunkBytes);
    const char *src = wg.pf_src;
    constexpr size_t kStep = (size_t)kWaves * kChunkBytes;
    uint32_t n;
    if (wg.pf_rem >= kStagePages) {
        n = kStagePages;
        dma_chunk(dst, src, lane_off);
        dma_chunk(dst + kChunkBytes, src + kStep, lane_off);
        dma_chunk(dst + 2 * kChunkBytes, src + 2 * kStep, lane_off);
        dma_chunk(dst + 3 * kChunkBytes, src + 3 * kStep, lane_off);
    } else {
        n = wg.pf_rem;
        dma_chunk(dst, src, lane_off);
        if (n > 1) dma_chunk(dst + kChunkBytes, src + kStep, lane_off);
        if (n > 2) dma_chunk(dst + 2 * kChunkBytes, src + 2 * kStep, lane_off);
    }
    wg.pf_src = src + n * kStep;
    wg.pf_rem -= n;
    wg.head += n;
    wg.hst = wg.hst + 1 == wg.nst ? 0 : wg.hst + 1;
}

// W4 tasks keep kPrefetchW4 chunks in flight per lane (their dequantisation is VALU work that more
// loads in flight cover); the scales that go with them are packed four to a slot behind the chunks.
constexpr int kPrefetchW4 = 12;
constexpr int kW4Slots = kPrefetchW4 + (kPrefetchW4 + 3) / 4;

constexpr int kBufSlots = kPrefetch > kW4Slots ? kPrefetch : kW4Slots;

struct GemvStream {
    const __attribute__((address_space(1))) u32x4 *wp;   // this lane's pointer to chunk 0 of the task
    uint32_t total;       // chunks in the task
    u32x4 buf[kBufSlots]; // direct-load path only: bf16 tasks use the first kPrefetch slots, W4 tasks kPrefetchW4 + scales
    const __attribute__((address_space(1))) uint16_t *sp;   // W4: this lane's scale of chunk 0 of the task
    uint32_t spc;                                            // W4: scales per chunk (2048 / group)
    // matrix-core W4 path: the scales of rows 4 ksub .. 4 ksub + 3 (four bf16 = 8 bytes) of each group of a chunk,
    // up to four groups (group size 32), fetched with the chunk
    u32x2 sbuf[kPrefetch][4];
};
__device__ __forceinline__ uint32_t w4_scale_get(const GemvStream &st, int j) { return st.buf[kPrefetchW4 + (j >> 2)][j & 3]; }
__device__ __forceinline__ void w4_scale_set(GemvStream &st, int j, uint32_t v) { st.buf[kPrefetchW4 + (j >> 2)][j & 3] = v; }

// Issue the first weight loads of a GEMV task.  They depend on nothing the
// previous operator produces, so this runs before the dependency wait.
template <bool RING, bool W4>
__device__ __forceinline__ void gemv_issue(const Params &P, const Instr &I, GemvStream &st, int npf)
{
    const int lane = threadIdx.x & 63, wave = (int)rfl(threadIdx.x >> 6);
    const bool sm = (I.flags & F_SLICE_MAJOR) != 0;
    const uint32_t groups = instr_groups(I);
    const uint32_t first = unit_chunk0(sm, I.u0, I.S, groups, I.kbt, I.nkb);
    const uint32_t end = unit_chunk0(sm, I.u0 + I.nu, I.S, groups, I.kbt, I.nkb);   // (one past the last unit)
    st.total = end - first;
    if (RING) return;
    st.wp = (const __attribute__((address_space(1))) u32x4 *)(uintptr_t)(P.ws + P.lay.weights) + ((size_t)I.w_chunk + first) * 64 + lane;
    const uint32_t last = st.total ? st.total - 1 : 0;
    const bool w4 = W4 && (I.flags & F_W4) != 0;
    if (w4) {
        // scale of this lane: group (32 ksub / group) of row r of the chunk, index g * R + r
        const uint32_t rlog = instr_rlog(I), R = 1u << rlog;
        const uint32_t sidx = (((uint32_t)lane >> rlog) * 32u / P.w4_group) * R + ((uint32_t)lane & (R - 1));
        st.spc = 2048u / P.w4_group;
        st.sp = (const __attribute__((address_space(1))) uint16_t *)(uintptr_t)(P.ws + P.lay.wscale) +
                ((size_t)I.w_chunk + first) * st.spc + sidx;
    }
    if (w4 && (I.flags & F_MFMA)) {
        // matrix-core form: 16 rows x 128 k per chunk; this lane's scales are rows 4 ksub .. + 3 of every group
        st.sp = (const __attribute__((address_space(1))) uint16_t *)(uintptr_t)(P.ws + P.lay.wscale) +
                ((size_t)I.w_chunk + first) * st.spc + 4u * ((uint32_t)lane >> 4);
        const uint32_t ngrp = 128u / P.w4_group;
#pragma unroll
        for (int j = 0; j < kPrefetch; ++j) {
            const uint32_t idx = min((uint32_t)wave + (uint32_t)j * kWaves, last);
            st.buf[j] = __builtin_nontemporal_load(st.wp + (size_t)idx * 64);
#pragma unroll
            for (int g = 0; g < 4; ++g)
                if ((uint32_t)g < ngrp) st.sbuf[j][g] = *(const __attribute__((address_space(1))) u32x2 *)(st.sp + (size_t)idx * st.spc + g * 16);
        }
        return;
    }
    if (w4) {
#pragma unroll
        for (int j = 0; j < kPrefetchW4; ++j) {
            uint32_t idx = min((uint32_t)wave + (uint32_t)j * kWaves, last);
            st.buf[j] = __builtin_nontemporal_load(st.wp + (size_t)idx * 64);
        }
#pragma unroll
        for (int j = 0; j < kPrefetchW4; ++j) {
            uint32_t idx = min((uint32_t)wave + (uint32_t)j * kWaves, last);
            w4_scale_set(st, j, st.sp[(size_t)idx * st.spc]);
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < kPrefetch; ++j) {
        if (j >= npf) continue;
        uint32_t idx = min((uint32_t)wave + (uint32_t)j * kWaves, last);
        st.buf[j] = __builtin_nontemporal_load(st.wp + (size_t)idx * 64);
    }
}

template <bool MFMA, bool RING, bool W4 = false>
__device__ __forceinline__ void gemv_main(const Params &P, const Instr &I, char *lds, Wg &lp, GemvStream &st, int batch)
{
    static_assert(!(W4 && RING), "W4 weights: direct loads only");
    const int tid = threadIdx.x, lane = tid & 63, wave = (int)rfl((uint32_t)tid >> 6);
    const uint32_t rlog = instr_rlog(I), R = 1u << rlog, ck = W4 ? chunk_k_w4(rlog) : chunk_k(rlog);
    const int ksub = lane >> rlog;
    char *xs = lds + lp.xs_off;
    float *red = (float *)(lds + kLdsRed);
    const int nterm = nterm_of(P.max_batch);
    const int ncols = MFMA ? batch * nterm : 1;
    const uint32_t S = I.S, nkb = I.nkb, kbt = I.kbt, nu = I.nu, u0 = I.u0;
    const uint32_t pro = instr_pro(I);
    const bool normk = (pro == PRO_EMBED_NORM || pro == PRO_RESID_NORM);
    const uint32_t x_kb0 = normk ? 0u : I.xs_lo;
    const uint32_t k_stage = normk ? (uint32_t)P.hidden : I.xs_hi * ck;
    const uint32_t plane_stride = k_stage * 2u + 16u;
    const uint32_t outs_per_unit = R * (uint32_t)(MFMA ? batch : 1);
    const uint32_t red_per_wave = nu * outs_per_unit;

    // running position of this wave inside the task: unit ul, chunk kbi within the unit
    uint32_t ul = 0, kbi = (uint32_t)wave;
    const bool sm = (I.flags & F_SLICE_MAJOR) != 0;
    const uint32_t groups = instr_groups(I);
    UnitCursor cur;
    unit_place(sm, u0, S, groups, cur.rg, cur.s);
    uint32_t cur_n = slice_chunks(cur.s, S, nkb, kbt);
    uint32_t cur_kb0 = cur.s * nkb;  // first chunk of the current unit inside its row group

    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    f32x4 cacc = {0.f, 0.f, 0.f, 0.f};    // matrix-core path: columns 0..15 (sequences 0..7, two terms each)
    f32x4 cacc2 = {0.f, 0.f, 0.f, 0.f};   //                   columns 16..31 (sequences 8..15), used when batch > 8
    const bool wide = MFMA && ncols > 16;

    auto flush = [&]() {
        if (!MFMA) {
            float v = (a0 + a1) + (a2 + a3);
            // Lanes sharing an output row differ in the lane bits >= rlog.  The bits inside a 16-lane
            // row are summed with DPP row rotations (by 8, 4, 2, 1: lanes congruent modulo R); the
            // four rows of the wave are NOT combined here -- each leaves its partial in its own slot
            // of the reduction area and the final fixed-order sum adds the 16 (wave, row) slots.
            // (A cross-row permute would stall the wave on the LDS crossbar at every unit.)
            if (R <= 8) v = dpp_add<0x128>(v);
            if (R <= 4) v = dpp_add<0x124>(v);
            if (R <= 2) v = dpp_add<0x122>(v);
            if (R <= 1) v = dpp_add<0x121>(v);
            if ((uint32_t)(lane & 15) < R) red[(wave * 4 + (lane >> 4)) * red_per_wave + ul * R + (lane & 15)] = v;
            a0 = a1 = a2 = a3 = 0.f;
        } else {
            // cacc[j] = C[row 4*ksub + j][col lane & 15]; sum the nterm columns of each sequence
            const int col = lane & 15;
#pragma unroll
            for (int grp = 0; grp < 2; ++grp) {
                if (grp && !wide) break;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float v = grp ? cacc2[j] : cacc[j];
                    // the term columns of a sequence are neighbours inside the 16-lane row: DPP row shifts
                    float v1 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x101, 0xf, 0xf, true));
                    float v2 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x102, 0xf, 0xf, true));
                    float sum = v + v1 + (nterm == 3 ? v2 : 0.f);
                    const int cc = col + 16 * grp, b = cc / nterm;
                    if (cc < ncols && cc == b * nterm)
                        red[wave * red_per_wave + (ul * batch + b) * 16 + ksub * 4 + j] = sum;
                }
            }
            cacc = f32x4{0.f, 0.f, 0.f, 0.f};
            cacc2 = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };

    // Matrix-core W4: one chunk = 16 rows x 128 k of codes.  Dword i of a lane holds the 8 codes of row lane % 16 for
    // k = 32 i + 8 ksub .. + 8, nibble p standing for k offset 2 (p % 4) + p / 4, so that (d >> 4 j) & 0x000f000f is the
    // pair (k 2j, k 2j + 1); OR-ing 0x4300 into each half makes the bf16 numbers 128 + q.  Four matrix-core
    // instructions per chunk; after the last one of a scale group the raw sums lose the zero point (136 times the
    // sum of the group's staged values, per column) and gain the scale.
    auto consume_w4m = [&](const u32x4 &w, const u32x2 (&sc)[4]) {
        while (kbi >= cur_n) {
            kbi -= cur_n;
            flush();
            ++ul;
            cur.next(sm, S, groups);
            cur_n = slice_chunks(cur.s, S, nkb, kbt);
            cur_kb0 = cur.s * nkb;
        }
        const uint32_t kb_rel = cur_kb0 + kbi - x_kb0;
        const int col = lane & 15;
        const bool live = col < ncols;
        const char *xk = xs + (size_t)col * plane_stride + ((size_t)kb_rel * 128u + (uint32_t)ksub * 8u) * 2u;
        const float *xsum = (const float *)(xs + (size_t)(P.max_batch * nterm) * plane_stride) + (size_t)col * (k_stage / 32u) + kb_rel * 4u;
        const uint32_t dw[4] = {w.x, w.y, w.z, w.w};
        const uint32_t group = P.w4_group;
        u32x4 xb[4];
        float zs[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {          // all LDS reads of the chunk first
            xb[i] = live ? *(const u32x4 *)(xk + i * 64) : u32x4{0u, 0u, 0u, 0u};
            zs[i] = live ? xsum[i] : 0.f;
        }
        f32x4 cg = {0.f, 0.f, 0.f, 0.f};
        float z = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t d = dw[i];
            u32x4 av;
            av.x = (d & 0x000f000fu) | 0x43004300u;
            av.y = ((d >> 4) & 0x000f000fu) | 0x43004300u;
            av.z = ((d >> 8) & 0x000f000fu) | 0x43004300u;
            av.w = ((d >> 12) & 0x000f000fu) | 0x43004300u;
            cg = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, xb[i]), cg, 0, 0, 0);
            z += zs[i];
            if (((uint32_t)(i + 1) * 32u) % group == 0u) {     // (wave-uniform) a scale group ends here
                const u32x2 sv = group == 32u ? sc[i] : group == 64u ? sc[i / 2] : sc[0];   // (static indices: the slots stay in registers)
                const float zp = 136.0f * z;
                cacc[0] += bf_lo(sv.x) * (cg[0] - zp); cacc[1] += bf_hi(sv.x) * (cg[1] - zp);
                cacc[2] += bf_lo(sv.y) * (cg[2] - zp); cacc[3] += bf_hi(sv.y) * (cg[3] - zp);
                cg = f32x4{0.f, 0.f, 0.f, 0.f};
                z = 0.f;
            }
        }
        kbi += kWaves;
    };

    auto consume = [&](const u32x4 &w, uint32_t sbits = 0) {
        // advance to the unit that holds this chunk, flushing finished units
        while (kbi >= cur_n) {
            kbi -= cur_n;
            flush();
            ++ul;
            cur.next(sm, S, groups);
            cur_n = slice_chunks(cur.s, S, nkb, kbt);
            cur_kb0 = cur.s * nkb;
        }
        const uint32_t kb_rel = cur_kb0 + kbi - x_kb0;  // chunk inside the staged vector
        if (W4) {
            // 32 codes of one row against 32 staged values: sum q x in fp32, then the zero point (8 times
            // the sum of the 32 values, precomputed by the prologue) and the group scale
            const uint32_t k0 = kb_rel * ck + (uint32_t)ksub * 32u;
            const f32x4 *xp = (const f32x4 *)(xs + (size_t)k0 * 4);
            const float *xsum = (const float *)(xs + (size_t)k_stage * 4);
            const uint32_t dw[4] = {w.x, w.y, w.z, w.w};
            float p0 = 0.f, p1 = 0.f, p2 = 0.f, p3 = 0.f;
            f32x4 xv[8];                                   // all eight LDS reads in flight before the arithmetic
#pragma unroll
            for (int i = 0; i < 8; ++i) xv[i] = xp[i];
            const float zsum = xsum[k0 >> 5];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t lo = dw[i] & 0x0f0f0f0fu, hi = (dw[i] >> 4) & 0x0f0f0f0fu;
                const f32x4 xa = xv[2 * i], xb = xv[2 * i + 1];
                p0 += ubyte_f<0>(lo) * xa.x; p1 += ubyte_f<0>(hi) * xa.y;
                p2 += ubyte_f<1>(lo) * xa.z; p3 += ubyte_f<1>(hi) * xa.w;
                p0 += ubyte_f<2>(lo) * xb.x; p1 += ubyte_f<2>(hi) * xb.y;
                p2 += ubyte_f<3>(lo) * xb.z; p3 += ubyte_f<3>(hi) * xb.w;
            }
            a0 += bf_to_f((uint16_t)sbits) * (((p0 + p1) + (p2 + p3)) - 8.0f * zsum);
        } else if (!MFMA) {
            const f32x4 *xp = (const f32x4 *)(xs + ((size_t)kb_rel * ck + ksub * 8) * 4);
            f32x4 x0 = xp[0], x1 = xp[1];
            a0 += bf_lo(w.x) * x0.x; a1 += bf_hi(w.x) * x0.y;
            a2 += bf_lo(w.y) * x0.z; a3 += bf_hi(w.y) * x0.w;
            a0 += bf_lo(w.z) * x1.x; a1 += bf_hi(w.z) * x1.y;
            a2 += bf_lo(w.w) * x1.z; a3 += bf_hi(w.w) * x1.w;
        } else {
            const int col = lane & 15;
            const char *xk = xs + ((size_t)kb_rel * ck + ksub * 8) * 2;
            u32x4 xb = {0u, 0u, 0u, 0u}, xb2 = {0u, 0u, 0u, 0u};
            if (col < ncols) xb = *(const u32x4 *)(xk + (size_t)col * plane_stride);
            if (wide && col + 16 < ncols) xb2 = *(const u32x4 *)(xk + (size_t)(col + 16) * plane_stride);
            bf16x8 av = __builtin_bit_cast(bf16x8, w);
            cacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, xb), cacc, 0, 0, 0);
            if (wide) cacc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, xb2), cacc2, 0, 0, 0);
        }
        kbi += kWaves;
    };

    // The residual row an F_ADD_RESID epilogue adds was final before this task's dependencies were
    // met: fetch the first (usually only) value of every thread now, one memory round trip earlier.
    float resid0 = 0.f;
    if (!MFMA && (I.flags & F_ADD_RESID) && (uint32_t)tid < red_per_wave) {
        const uint32_t ub = (uint32_t)tid >> rlog, uu = u0 + ub;
        uint32_t rg, s;
        unit_place(sm, uu, S, groups, rg, s);
        resid0 = ld_act((const float *)(P.scr + P.lay.act) + I.resid + (size_t)rg * R + ((uint32_t)tid & (R - 1)));
    }
    // Likewise the bias of this thread's first output (a constant).
    float bias0 = 0.f;
    if (I.bias != kNone && (uint32_t)tid < red_per_wave) {
        const uint32_t nb0 = (uint32_t)(MFMA ? batch : 1);
        const uint32_t uu = u0 + ((uint32_t)tid >> rlog) / nb0;
        uint32_t rg, s;
        unit_place(sm, uu, S, groups, rg, s);
        const uint32_t row = rg * R + ((uint32_t)tid & (R - 1));
        if (s == 0 && row < I.n_rows) bias0 = bf_to_f(((const uint16_t *)(P.ws + P.lay.vecs))[I.bias + row]);
    }
    const uint32_t total = st.total;
    if (RING) {
        // Weights come from this wave's LDS page ring, a stage (up to four chunks) at a time:
        // wait until the stage's DMA loads have landed (loads complete in issue order, so "at most
        // head - tail - n outstanding" means the n oldest chunks are there), read it back, hand the
        // stage to the DMA again as soon as the reads have returned, and use the registers while
        // the next stage is being read.
        const uint32_t mine = total > (uint32_t)wave ? (total - (uint32_t)wave + kWaves - 1) / kWaves : 0u;
        const uint32_t ng = (mine + kStagePages - 1) / kStagePages;
        const char *ring = lds + lp.ring_off + lane * 16;
        bool ok = true;
        // n == 0: no further stage of this task -- the registers are still (re)defined by in-bounds
        // reads whose values are never used, which keeps them free of loop-carried copies
        auto read_stage = [&](u32x4 (&w)[kStagePages], uint32_t n) {
            if (n) {
                const uint32_t out = lp.head - lp.tail;
                if (out < n) {   // stream table and instruction list disagree: never use an unfilled page
                    set_err(P, 2, 1u);
                    ok = false;
                } else {
                    vm_wait4((out - n) >> 2);
                }
            }
            const char *base = ring + (size_t)lp.tst * (kStagePages * kChunkBytes);
#pragma unroll
            for (uint32_t u = 0; u < kStagePages; ++u) w[u] = *(const u32x4 *)(base + u * kChunkBytes);
            if (n) {
                lp.tail += n;
                lp.tst = lp.tst + 1 == lp.nst ? 0 : lp.tst + 1;
            }
        };
        auto step = [&](u32x4 (&wc)[kStagePages], u32x4 (&wn)[kStagePages], uint32_t g) {
            const uint32_t n = g < ng ? min(kStagePages, mine - g * kStagePages) : 0u;
            // the reads of this stage have returned: its pages go back to the DMA
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (n) ring_fill_stage(P, lp);
            read_stage(wn, g + 1 < ng ? min(kStagePages, mine - (g + 1) * kStagePages) : 0u);
#pragma unroll
            for (uint32_t u = 0; u < kStagePages; ++u)
                if (u < n && ok) consume(wc[u]);
        };
        u32x4 w0[kStagePages], w1[kStagePages];
        read_stage(w0, min(kStagePages, mine));
        for (uint32_t g = 0; g < ng; g += 2) {
            step(w0, w1, g);
            step(w1, w0, g + 1);
        }
    } else if (W4 && MFMA) {
        if (total) {
            const uint32_t last = total - 1, ngrp = 128u / P.w4_group;
            constexpr uint32_t round = (uint32_t)kPrefetch * kWaves;
            uint32_t base = 0;
            for (; base + round < total; base += round) {
#pragma unroll
                for (int j = 0; j < kPrefetch; ++j) {
                    const uint32_t idx = base + (uint32_t)j * kWaves + (uint32_t)wave;
                    consume_w4m(st.buf[j], st.sbuf[j]);
                    const uint32_t nidx = min(idx + round, last);
                    st.buf[j] = __builtin_nontemporal_load(st.wp + (size_t)nidx * 64);
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        if ((uint32_t)g < ngrp) st.sbuf[j][g] = *(const __attribute__((address_space(1))) u32x2 *)(st.sp + (size_t)nidx * st.spc + g * 16);
                }
            }
#pragma unroll
            for (int j = 0; j < kPrefetch; ++j) {
                const uint32_t idx = base + (uint32_t)j * kWaves + (uint32_t)wave;
                if (idx < total) consume_w4m(st.buf[j], st.sbuf[j]);
            }
        }
    } else if (W4) {
        // Rounds of kPrefetchW4 slots per wave: a slot is consumed, then refilled with the chunk one round
        // ahead.  The last round refills nothing, so no load is outstanding when the task ends (the
        // store drain before the task's signal would wait for it).
        if (total) {
            const uint32_t last = total - 1;
            constexpr uint32_t round = (uint32_t)kPrefetchW4 * kWaves;
            uint32_t base = 0;
            for (; base + round < total; base += round) {
#pragma unroll
                for (int j = 0; j < kPrefetchW4; ++j) {
                    const uint32_t idx = base + (uint32_t)j * kWaves + (uint32_t)wave;
                    consume(st.buf[j], w4_scale_get(st, j));
                    const uint32_t nidx = min(idx + round, last);
                    st.buf[j] = __builtin_nontemporal_load(st.wp + (size_t)nidx * 64);
                    w4_scale_set(st, j, st.sp[(size_t)nidx * st.spc]);
                }
            }
#pragma unroll
            for (int j = 0; j < kPrefetchW4; ++j) {
                const uint32_t idx = base + (uint32_t)j * kWaves + (uint32_t)wave;
                if (idx < total) consume(st.buf[j], w4_scale_get(st, j));
            }
        }
    } else if (total) {
        const uint32_t last = total - 1;
        const uint32_t round = (uint32_t)lp.npf * kWaves;
        uint32_t base = 0;
        for (; base + round < total; base += round) {
#pragma unroll
            for (int j = 0; j < kPrefetch; ++j) {
                if (j >= lp.npf) continue;
                const uint32_t idx = base + (uint32_t)j * kWaves + (uint32_t)wave;
                consume(st.buf[j]);
                // refill the slot: always a load (clamped to the task's last chunk), so the slot's
                // registers are written by exactly one instruction and nothing waits on it here
                const uint32_t nidx = min(idx + round, last);
                st.buf[j] = __builtin_nontemporal_load(st.wp + (size_t)nidx * 64);
            }
        }
        // last round: nothing to refill, so no load is outstanding when the task ends (the store
        // drain before the task's signal would wait for it)
#pragma unroll
        for (int j = 0; j < kPrefetch; ++j) {
            if (j >= lp.npf) continue;
            const uint32_t idx = base + (uint32_t)j * kWaves + (uint32_t)wave;
            if (idx < total) consume(st.buf[j]);
        }
    }
    // flush the current unit and any trailing units this wave had no chunk in
    while (ul < nu) {
        flush();
        ++ul;
    }
    wg_sync(lp, lds);
    if ((P.flags & 1u) && tid == 0 && P.only_seq == kNone)   // task trace, mark 3: weights consumed, partial sums in LDS
        ((uint64_t *)(P.ws + P.lay.trace))[((size_t)blockIdx.x * P.max_instr + lp.pc) * 8 + 7] = wall_clock64();

    // cross-wave sum in fixed wave order, then the epilogue
    const ActBuf ab = act_buf(P);
    float *actw = (float *)(P.scr + P.lay.act);
    const uint32_t nb = (uint32_t)(MFMA ? batch : 1);
    auto rsum = [&](uint32_t t) {
        constexpr int kSlots = MFMA ? kWaves : kWaves * 4;   // VALU path: one slot per (wave, 16-lane row)
        float p[kSlots];                                     // all LDS reads first, then the sum in slot order
#pragma unroll
        for (int w = 0; w < kSlots; ++w) p[w] = red[w * red_per_wave + t];
        float v = p[0];
#pragma unroll
        for (int w = 1; w < kSlots; ++w) v += p[w];
        return v;
    };
    if (I.flags & F_SILU_EPI) {
        // row group = R/2 gate rows then R/2 up rows; out[group * R/2 + r] = silu(gate) * up
        const uint32_t half = R >> 1, nout = nu * nb * half;
        for (uint32_t t = tid; t < nout; t += kWgThreads) {
            uint32_t r = t % half, ub = t / half;
            float g = rsum(ub * R + r), u = rsum(ub * R + half + r);
            uint32_t b = ub % nb, uu = u0 + ub / nb;
            uint32_t row = uu * half + r;     // S == 1: unit index == row group
            st_act(actw + I.out + (size_t)b * I.out_ld + row, g / (1.0f + __expf(-g)) * u);
        }
    } else {
        for (uint32_t t = tid; t < red_per_wave; t += kWgThreads) {
            float v = rsum(t);
            uint32_t r = t & (R - 1), ub = t >> rlog;
            uint32_t b = ub % nb, uu = u0 + ub / nb;
            uint32_t rg, s;
            unit_place(sm, uu, S, groups, rg, s);
            uint32_t row = rg * R + r;
            if (I.bias != kNone && s == 0 && row < I.n_rows)
                v += t == (uint32_t)tid ? bias0 : bf_to_f(((const uint16_t *)(P.ws + P.lay.vecs))[I.bias + row]);
            if (I.flags & F_LOGITS) {
                if (row < I.n_rows) lp.logits[(size_t)b * P.vocab + row] = v;
                // this thread is the only reader of index t of the reduction area: keep the finished
                // logit there for the arg-max pass below
                if ((I.flags & F_ARGMAX) && P.want_tokens) red[t] = row < I.n_rows ? v : -INFINITY;
            } else {
                if (I.flags & F_ADD_RESID) v += (!MFMA && t == (uint32_t)tid) ? resid0 : ld_act(actw + I.resid + (size_t)b * I.out_ld + row);
                st_act(actw + I.out + (size_t)s * I.out_split_stride + (size_t)b * I.out_ld + row, v);
            }
        }
        if ((I.flags & F_ARGMAX) && P.want_tokens) {
            // (max logit, its row) of this task per sequence; ties go to the smaller row
            float *sv = (float *)(lds + kLdsMisc + 64);
            uint32_t *si = (uint32_t *)(lds + kLdsMisc + 80);
            for (uint32_t b = 0; b < nb; ++b) {
                wg_sync(lp, lds);
                float bv = -INFINITY;
                uint32_t bi = 0xffffffffu;
                for (uint32_t t = tid; t < red_per_wave; t += kWgThreads) {
                    const uint32_t ub = t >> rlog;
                    if (ub % nb != b) continue;
                    const float v = red[t];
                    const uint32_t row = (u0 + ub / nb) * R + (t & (R - 1));   // (the LM head has one K slice: unit = row group)
                    if (v > bv || (v == bv && row < bi)) { bv = v; bi = row; }
                }
                argmax_wave(bv, bi);
                if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
                wg_sync(lp, lds);
                if (tid == 0) {
                    for (int w = 1; w < kWaves; ++w)
                        if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
                    float *dst = actw + P.amax + ((size_t)I.spare * P.max_batch + b) * 2;
                    st_act(dst, bv);
                    st_act(dst + 1, __uint_as_float(bi));
                }
            }
        }
    }
    (void)ab;
}

// Task-internal trace mark k (0..3) of instruction pc; compiled to nothing unless tracing.
__device__ __forceinline__ void trace_mark(const Params &P, uint32_t pc, int k)
{
    if ((P.flags & 1u) && threadIdx.x == 0 && P.only_seq == kNone)
        ((uint64_t *)(P.ws + P.lay.trace))[((size_t)blockIdx.x * P.max_instr + pc) * 8 + 4 + k] = wall_clock64();
}

// ---------------------------------------------------------------- attention task
// Flash-decode partial over the history positions owned by chunk task c of
// (sequence b, kv head g): blocks c, c+nc, c+2nc, ... of `bs` positions.  All
// q heads of the group are processed against each K/V row read once.  The
// task that owns the block of the current position also rotates/rounds the
// new k and v, appends them to the cache and attends to them from LDS.
//
// The K/V history does not depend on this step's QKV projection, so the first
// loads of the task are issued before the dependency wait (paper Sec. 4.2.3,
// Fig. 4: history KV loads leave the critical path).
template <int GM>
struct AttState {
    float m[GM], l[GM];
    float acc[GM][8];
};

constexpr int kAttPrefetch = 6;   // K and V 128-bit loads in flight per lane
constexpr int kPartStride = 4;    // partial rows are [acc[D], m, l, pad, pad] so that they stay 16-byte aligned

struct AttStream {
    const __attribute__((address_space(1))) u32x4 *kp, *vp;   // this lane's K / V row base (position 0, own 8-dim slice)
    int p, npos, sub;
    u32x4 kbuf[kAttPrefetch], vbuf[kAttPrefetch];
};

__device__ __forceinline__ float safe_exp_diff(float a, float M)
{
    return (a == -INFINITY) ? 0.f : __expf(a - M);
}

// position (in the cache) of flattened index idx of task c; blocks are kAttBlock = 16 positions
constexpr int kAttBlockLog = 4;
__device__ __forceinline__ int att_pos(int idx, int bs, int nc, int c)
{
    (void)bs;
    const int blk = idx >> kAttBlockLog;
    return ((c + blk * nc) << kAttBlockLog) + (idx & ((1 << kAttBlockLog) - 1));
}

template <int D>
__device__ __forceinline__ void att_issue(const Params &P, const Wg &lp, const InstrAtt &I, AttStream &st)
{
    constexpr int LPP = D / 8, PPW = 64 / LPP;
    typedef const __attribute__((address_space(1))) u32x4 *gp;
    const int lane = threadIdx.x & 63, wave = (int)rfl(threadIdx.x >> 6);
    const int b = (int)I.b, g = (int)I.g;
    st.npos = 0; st.p = 0; st.sub = lane / LPP;
    if (b >= P.batch) return;
    const int p = position_of(P, lp, b);
    const int bs = (int)I.bs, nc = (int)I.nc, c = (int)I.c;
    const int nblk_all = (p + bs) >> kAttBlockLog;                // blocks containing positions <= p (the new one included)
    const int my_blocks = (nblk_all > c) ? (nblk_all - c + nc - 1) / nc : 0;
    st.p = p; st.npos = my_blocks * bs;
    const size_t head_elems = (size_t)P.max_context * D;
    const uint16_t *Kc = P.kv + ((((size_t)I.layer * 2 + 0) * P.max_batch + b) * P.n_kv_heads + g) * head_elems;
    const uint16_t *Vc = P.kv + ((((size_t)I.layer * 2 + 1) * P.max_batch + b) * P.n_kv_heads + g) * head_elems;
    st.kp = (gp)(uintptr_t)Kc + (lane % LPP);
    st.vp = (gp)(uintptr_t)Vc + (lane % LPP);
#pragma unroll
    for (int j = 0; j < kAttPrefetch; ++j) {
        const int grp = (wave + j * kWaves) * PPW;
        // Rows at or beyond p are masked when consumed; their loads go to the last history row instead,
        // so that no cache ever holds a line of a row before the step that appends it has written it
        // (steps of one launch follow each other without a cache invalidate).
        int t = att_pos(grp + st.sub, bs, nc, c);
        t = t < p ? t : p - 1;
        st.kbuf[j] = u32x4{0u, 0u, 0u, 0u};
        st.vbuf[j] = u32x4{0u, 0u, 0u, 0u};
        if (grp < st.npos && p > 0) {
            st.kbuf[j] = __builtin_nontemporal_load(st.kp + (size_t)t * LPP);
            st.vbuf[j] = __builtin_nontemporal_load(st.vp + (size_t)t * LPP);
        }
    }
}

// Prologue of an attention task (both forms): the q heads of the task -- and, in the task that owns the block of the
// new position, the new k and v -- are summed from the QKV partials, normalised (QK-norm), rotated and left in LDS:
// sq [kMaxGroup][D] (pre-scaled by 1/sqrt(D)), snew [2][D] (rounded to bf16 like the rows in the cache).  The owner of
// the group's first heads appends the new rows to the cache.  Returns whether this task owns the new position.
template <int D>
__device__ __forceinline__ bool att_prologue(const Params &P, const InstrAtt &I, char *lds, Wg &lp, int p, uint32_t pc)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = (int)rfl((uint32_t)tid >> 6);
    const int b = (int)I.b, g = (int)I.g;
    // The task covers heads [hb, hb + G) of the GG query heads that share KV head g.
    const int GG = P.n_q_heads / P.n_kv_heads, hb = (int)I.h0, G = (int)I.nh;
    const int qd = P.n_q_heads * D, kvd = P.n_kv_heads * D;
    const float *act = (const float *)(P.scr + P.lay.act);
    const uint16_t *vecs = (const uint16_t *)(P.ws + P.lay.vecs);
    const float *rope = (const float *)(P.ws + P.lay.rope) + (size_t)p * D;  // [D/2][2]
    float *sq = (float *)(lds + lp.xs_off);
    float *snew = sq + kMaxGroup * D;
    const int jb_new = p >> kAttBlockLog;
    const bool owner = (jb_new % (int)I.nc) == (int)I.c;

    // ---- prologue: q heads (and new k / v) : sum partials, optional RMSNorm, RoPE
    const int nvec = G + (owner ? 2 : 0);
    // Each wave owns vectors wave, wave+4, wave+8 (q heads, then new k, then new v).  All their
    // loads are issued before any is used, so the prologue costs one memory round trip.
    constexpr int kRounds = (kMaxGroup + 2 + kWaves - 1) / kWaves;
    float pa[kRounds], pb[kRounds];
    const int i = lane;   // pair index (i, i + D/2)
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int vi = wave + r * kWaves;
        pa[r] = 0.f; pb[r] = 0.f;
        if (vi < nvec && i < D / 2) {
            const int row0 = vi < G ? (g * GG + hb + vi) * D : (vi == G ? qd + g * D : qd + kvd + g * D);
            for (uint32_t s = 0; s < I.n_parts; ++s) {
                const float *pp = act + I.in_parts + (size_t)s * I.part_stride + (size_t)b * I.in_ld + row0;
                float u0 = ld_act(pp + i), u1 = ld_act(pp + i + D / 2);
                pa[r] += u0;
                pb[r] += u1;
            }
        }
    }
    float cs = 0.f, sn = 0.f;
    if (i < D / 2) { cs = rope[2 * i]; sn = rope[2 * i + 1]; }
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int vi = wave + r * kWaves;
        if (vi >= nvec) continue;
        const bool rot = vi <= G;
        const uint32_t gain_off = vi < G ? I.qn_gain : I.kn_gain;
        float a = pa[r], c2 = pb[r];
        if (rot) {
            if (P.qk_norm && gain_off != kNone) {
                float ss = wave_sum(a * a + c2 * c2);
                float inv = 1.0f / sqrtf(ss / (float)D + P.rms_eps);
                if (i < D / 2) {
                    a = a * inv * bf_to_f(vecs[gain_off + i]);
                    c2 = c2 * inv * bf_to_f(vecs[gain_off + i + D / 2]);
                }
            }
            float ra = a * cs - c2 * sn;
            float rb = c2 * cs + a * sn;
            a = ra; c2 = rb;
        }
        if (i < D / 2) {
            if (vi < G) {
                const float scale = 1.0f / sqrtf((float)D);
                sq[vi * D + i] = a * scale;
                sq[vi * D + i + D / 2] = c2 * scale;
            } else {
                const int which = vi - G;  // 0 = K, 1 = V
                snew[which * D + i] = bf_to_f(f_to_bf(a));
                snew[which * D + i + D / 2] = bf_to_f(f_to_bf(c2));
            }
        }
    }
    wg_sync(lp, lds);
    trace_mark(P, pc, 0);
    // append the new K and V rows (bf16 pairs, write-through: the next step of the same launch reads them)
    if (owner && hb == 0 && tid < D) {   // (of the tasks that share this chunk, the one with the group's first heads appends)
        typedef __attribute__((address_space(1))) uint32_t *gptr;
        const int which = tid / (D / 2), j = tid % (D / 2);
        const size_t base = ((((size_t)I.layer * 2 + which) * P.max_batch + b) * P.n_kv_heads + g) *
                                (size_t)P.max_context * D + (size_t)p * D;
        // (the staged values are already rounded to bf16: their upper halves are the codes)
        const uint32_t pk = (__float_as_uint(snew[which * D + 2 * j]) >> 16) | (__float_as_uint(snew[which * D + 2 * j + 1]) & 0xffff0000u);
        __hip_atomic_store((gptr)(uintptr_t)(P.kv + base + 2 * j), pk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return owner;
}

// GM: the most heads a task may carry (its running states and q slices live in registers, sized by GM whatever the task's
// own head count: tasks of at most four heads run the GM = 4 form, which leaves the register file room to spare).
template <int D, int GM>
__device__ __forceinline__ void att_task(const Params &P, const InstrAtt &I, char *lds, Wg &lp, AttStream &as, uint32_t pc)
{
    constexpr int LPP = D / 8;       // lanes per position (16 B each)
    constexpr int PPW = 64 / LPP;    // positions per wavefront load
    const int tid = threadIdx.x, lane = tid & 63, wave = (int)rfl((uint32_t)tid >> 6);
    const int b = (int)I.b, g = (int)I.g;
    if (b >= P.batch) return;
    const int GG = P.n_q_heads / P.n_kv_heads, hb = (int)I.h0, G = (int)I.nh;
    const int p = as.p;

    // LDS scratch inside the xs region
    float *sq = (float *)(lds + lp.xs_off);              // [G][D] rotated, pre-scaled q
    float *snew = sq + kMaxGroup * D;                    // [2][D] new k (rotated, bf16-rounded) and v
    float *smerge = snew + 2 * D;                        // [kWaves * PPW][G][MS]: acc[D], m, l, pad (rows 16-byte aligned)
    constexpr int MS = D + 4;
    const bool owner = att_prologue<D>(P, I, lds, lp, p, pc);

    // ---- main loop over this task's history positions (t < p)
    const int sub = as.sub, dl = lane % LPP;   // position inside the load, 8-dim slice
    AttState<GM> st;
#pragma unroll
    for (int h = 0; h < GM; ++h) {
        st.m[h] = -INFINITY; st.l[h] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) st.acc[h][j] = 0.f;
    }
    const int bs = (int)I.bs, nc = (int)I.nc, c = (int)I.c;
    const int npos = as.npos;

    // this lane's 8-dim slice of every (rotated, pre-scaled) q head, read from LDS once
    f32x4 qreg[GM][2];
#pragma unroll
    for (int h = 0; h < GM; ++h) {
        const f32x4 *qp = (const f32x4 *)(sq + (h < G ? h : 0) * D + dl * 8);
        qreg[h][0] = qp[0];
        qreg[h][1] = qp[1];
    }

    // Online softmax over batches of up to three positions per lane group: one running-max update and
    // one rescale of the accumulators per batch instead of per position (wave64 VALU ops cost four
    // cycles each, and this loop is VALU-bound).  N = positions actually present in the batch.
    auto batchN = [&](auto nn, const u32x4 &k0, const u32x4 &v0, bool ok0, const u32x4 &k1, const u32x4 &v1, bool ok1,
                      const u32x4 &k2, const u32x4 &v2, bool ok2) {
        constexpr int N = decltype(nn)::value;
        const u32x4 kw[3] = {k0, k1, k2};
        const u32x4 vw[3] = {v0, v1, v2};
        const bool ok[3] = {ok0, ok1, ok2};
        float vf[N][8];
#pragma unroll
        for (int u = 0; u < N; ++u) {
            // a masked position contributes exactly zero whatever its (possibly never written) row holds
            const u32x4 vv = ok[u] ? vw[u] : u32x4{0u, 0u, 0u, 0u};
            vf[u][0] = bf_lo(vv.x); vf[u][1] = bf_hi(vv.x); vf[u][2] = bf_lo(vv.y); vf[u][3] = bf_hi(vv.y);
            vf[u][4] = bf_lo(vv.z); vf[u][5] = bf_hi(vv.z); vf[u][6] = bf_lo(vv.w); vf[u][7] = bf_hi(vv.w);
        }
#pragma unroll
        for (int h = 0; h < GM; ++h)
            if (h < G) {
                const f32x4 q0 = qreg[h][0], q1 = qreg[h][1];
                float sc[N];
                float mn = st.m[h];
#pragma unroll
                for (int u = 0; u < N; ++u) {
                    float d = q0.x * bf_lo(kw[u].x) + q0.y * bf_hi(kw[u].x) + q0.z * bf_lo(kw[u].y) + q0.w * bf_hi(kw[u].y) +
                              q1.x * bf_lo(kw[u].z) + q1.y * bf_hi(kw[u].z) + q1.z * bf_lo(kw[u].w) + q1.w * bf_hi(kw[u].w);
                    d = (LPP == 16) ? row_sum16(d) : row_sum8(d);
                    sc[u] = ok[u] ? d : -INFINITY;
                    mn = fmaxf(mn, sc[u]);
                }
                const float rs = safe_exp_diff(st.m[h], mn);
                float pr[N], psum = 0.f;
#pragma unroll
                for (int u = 0; u < N; ++u) { pr[u] = safe_exp_diff(sc[u], mn); psum += pr[u]; }
                st.l[h] = st.l[h] * rs + psum;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    float a = pr[0] * vf[0][j];
#pragma unroll
                    for (int u = 1; u < N; ++u) a += pr[u] * vf[u][j];
                    st.acc[h][j] = st.acc[h][j] * rs + a;
                }
                st.m[h] = mn;
            }
    };
    static_assert(kAttPrefetch % 3 == 0, "the prefetch slots are consumed three at a time");
    // The new position p sits in the owner task's last block like any history position; its K and V
    // rows come from LDS (this lane's 8-dim slice, bf16-rounded like the rows in the cache) instead
    // of from the load, which went to row p - 1.
    u32x4 knew = {0u, 0u, 0u, 0u}, vnew = {0u, 0u, 0u, 0u};
    if (owner) {
        const float *kn = snew + dl * 8, *vn = snew + D + dl * 8;
        auto pair = [](float lo, float hi) { return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xffff0000u); };
        const f32x4 k0 = *(const f32x4 *)kn, k1 = *(const f32x4 *)(kn + 4), v0 = *(const f32x4 *)vn, v1 = *(const f32x4 *)(vn + 4);
        knew = u32x4{pair(k0.x, k0.y), pair(k0.z, k0.w), pair(k1.x, k1.y), pair(k1.z, k1.w)};
        vnew = u32x4{pair(v0.x, v0.y), pair(v0.z, v0.w), pair(v1.x, v1.y), pair(v1.z, v1.w)};
    }

    for (int base = 0; base * PPW < npos; base += kAttPrefetch * kWaves) {
#pragma unroll
        for (int j0 = 0; j0 < kAttPrefetch; j0 += 3) {
            if ((base + wave + j0 * kWaves) * PPW < npos) {   // (wave-uniform) this batch has at least one group
                bool ok[3];
                u32x4 kk[3], vv[3];
#pragma unroll
                for (int u = 0; u < 3; ++u) {
                    const int grp = (base + wave + (j0 + u) * kWaves) * PPW;
                    const int t = att_pos(grp + sub, bs, nc, c);
                    ok[u] = grp < npos && t <= p;
                    const bool fresh = t == p;        // only ever true in the owner task
                    kk[u] = fresh ? knew : as.kbuf[j0 + u];
                    vv[u] = fresh ? vnew : as.vbuf[j0 + u];
                }
                batchN(std::integral_constant<int, 3>{}, kk[0], vv[0], ok[0], kk[1], vv[1], ok[1], kk[2], vv[2], ok[2]);
            }
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                const int ngrp = (base + wave + (j0 + u) * kWaves) * PPW + kAttPrefetch * kWaves * PPW;
                if (ngrp < npos) {   // (a second round implies p > 0)
                    int t = att_pos(ngrp + sub, bs, nc, c);
                    t = t < p ? t : p - 1;
                    as.kbuf[j0 + u] = __builtin_nontemporal_load(as.kp + (size_t)t * LPP);
                    as.vbuf[j0 + u] = __builtin_nontemporal_load(as.vp + (size_t)t * LPP);
                }
            }
        }
    }

    trace_mark(P, pc, 1);
    // ---- every (wave, position slot) leaves its running state in LDS; merged below in fixed order
    constexpr int NSLOT = kWaves * PPW;
    {
        const int slot = wave * PPW + sub;
#pragma unroll
        for (int h = 0; h < GM; ++h)
            if (h < G) {
                float *dst = smerge + ((size_t)slot * G + h) * MS;
                f32x4 lo4 = {st.acc[h][0], st.acc[h][1], st.acc[h][2], st.acc[h][3]};
                f32x4 hi4 = {st.acc[h][4], st.acc[h][5], st.acc[h][6], st.acc[h][7]};
                *(f32x4 *)(dst + dl * 8) = lo4;
                *(f32x4 *)(dst + dl * 8 + 4) = hi4;
                if (dl == 0) { dst[D] = st.m[h]; dst[D + 1] = st.l[h]; }
            }
    }
    wg_sync(lp, lds);
    trace_mark(P, pc, 2);

    // merged max, denominator and per-slot weights of every head: thread (head, slot), the slots of a
    // head in adjacent lanes (NSLOT is 16 or 32, so rows of 16 lanes are all active or all idle)
    float *sfac = smerge + (size_t)NSLOT * G * MS;     // [G][NSLOT] weights, then [G] max, [G] denominators
    static_assert(NSLOT == 16 || NSLOT == 32, "slot reduction works on rows of 16 lanes");
    if (tid < G * NSLOT) {
        const int h = tid / NSLOT, w = tid % NSLOT;
        const float *src = smerge + ((size_t)w * G + h) * MS;
        const float m = src[D], l = src[D + 1];
        float M = row_max16(m);
        if (NSLOT == 32) M = fmaxf(M, __shfl_xor(M, 16, 64));
        const float f = safe_exp_diff(m, M);
        float L = row_sum16(f * l);
        if (NSLOT == 32) L += __shfl_xor(L, 16, 64);
        sfac[h * NSLOT + w] = f;
        if (w == 0) { sfac[G * NSLOT + h] = M; sfac[G * NSLOT + G + h] = L; }
    }
    wg_sync(lp, lds);
    const ActBuf ab = act_buf(P);
    for (int e = tid; e < G * D / 4; e += kWgThreads) {       // four adjacent outputs per thread
        const int h = (4 * e) / D, i = (4 * e) % D;
        // all LDS reads first, then the sums in slot order (the reads overlap instead of each waiting for the last)
        f32x4 sv[NSLOT];
        float fv[NSLOT];
#pragma unroll
        for (int w = 0; w < NSLOT; ++w) {
            sv[w] = *(const f32x4 *)(smerge + ((size_t)w * G + h) * MS + i);
            fv[w] = sfac[h * NSLOT + w];
        }
        f32x4 A = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NSLOT; ++w) A += sv[w] * fv[w];
        // partial layout [b][head][nc][D + kPartStride]
        const uint32_t dst = I.out + (uint32_t)((((size_t)b * P.n_q_heads + (g * GG + hb + h)) * I.nc + I.c) * (D + kPartStride));
        st_act4(ab, dst + (uint32_t)i, A);
        if (i == 0) {
            float *ml = (float *)(P.scr + P.lay.act) + dst + D;
            st_act(ml, sfac[G * NSLOT + h]);
            st_act(ml + 1, sfac[G * NSLOT + G + h]);
        }
    }
    trace_mark(P, pc, 3);
}

// ---------------------------------------------------------------- attention task on the matrix cores
// The same flash-decode partial as att_task, for the kernels that serve several sequences: there the history loop of
// the vector form is bound by its arithmetic (every lane of a 16-lane group repeats the soft-max bookkeeping of
// each head), not by the K/V stream.  Here a wavefront takes whole blocks of 16 positions:
//   scores   S[pos][col] = K[pos][:] . q[col][:]       D/32 x v_mfma_f32_16x16x32_bf16; the K rows are the A operand
//            straight from the cache (lane % 16 = position, lane / 16 = 16-byte slice of every 64 bytes of the row),
//            the B operand holds the rotated, pre-scaled q of every head as TWO bf16 columns (hi, lo), so that
//            the product keeps fp32-like accuracy: up to 8 heads fill the 16 columns;
//   soft-max once per (position, column): a lane owns four positions of one column; the running maximum of a
//            column is only raised when some score of the block exceeds it (a wave-wide vote), and only then are the
//            accumulators rescaled;
//   values   O^T[d][col] += V^T[d][pos] . P[pos][col]  D/16 x v_mfma_f32_16x16x16_bf16; P is again hi / lo columns and is
//            already laid out as the B operand (a lane's four positions are its four k values); V^T comes from a
//            transposed copy of the block in LDS (rows of 16 positions), written with 16-bit stores.
// Each wavefront leaves (max, denominator, accumulators) per head in LDS; they are merged in wave order and stored in
// the same partial-row format as att_task writes, so that combine tasks and the fused combine read either.
constexpr int kAttMcDepth = 2;   // blocks (K and V rows of 16 positions) a wavefront keeps in flight
constexpr int kVtRow = 40;       // bytes per row of the transposed V block: 16 positions of bf16 + 8 bytes of bank skew
typedef short s16x4 __attribute__((ext_vector_type(4)));

template <int D>
struct AttStreamMc {
    const __attribute__((address_space(1))) u32x4 *kp, *vp;   // K / V of (sequence, kv head): row 0, this lane's 16-byte slice
    int p, nblk;                                               // position of the new token; blocks of this wavefront
    u32x4 kbuf[kAttMcDepth][D / 32], vbuf[kAttMcDepth][D / 32];
};

// Loads of block kk of this wavefront (blocks wave, wave + 4, ... of the task) into slot s.  Rows at or beyond p go
// to row p - 1 instead (they are masked when consumed): no cache then holds a line of a row before the step that
// appends it has written it.
template <int D>
__device__ __forceinline__ void att_mc_load(const InstrAtt &I, AttStreamMc<D> &st, int s, int kk)
{
    const int lane = threadIdx.x & 63, wave = (int)rfl(threadIdx.x >> 6);
    int t = (((int)I.c + (wave + kk * kWaves) * (int)I.nc) << kAttBlockLog) + (lane & 15);
    t = t < st.p ? t : st.p - 1;
#pragma unroll
    for (int i = 0; i < D / 32; ++i) {
        st.kbuf[s][i] = __builtin_nontemporal_load(st.kp + (size_t)t * (D / 8) + 4 * i);
        st.vbuf[s][i] = __builtin_nontemporal_load(st.vp + (size_t)t * (D / 8) + 4 * i);
    }
}

template <int D>
__device__ __forceinline__ void att_issue_mc(const Params &P, const Wg &lp, const InstrAtt &I, AttStreamMc<D> &st)
{
    typedef const __attribute__((address_space(1))) u32x4 *gp;
    const int lane = threadIdx.x & 63, wave = (int)rfl(threadIdx.x >> 6);
    const int b = (int)I.b, g = (int)I.g;
    st.p = 0; st.nblk = 0;
#pragma unroll
    for (int s = 0; s < kAttMcDepth; ++s)
#pragma unroll
        for (int i = 0; i < D / 32; ++i) { st.kbuf[s][i] = u32x4{0u, 0u, 0u, 0u}; st.vbuf[s][i] = u32x4{0u, 0u, 0u, 0u}; }
    if (b >= P.batch) return;
    const int p = position_of(P, lp, b);
    const int nc = (int)I.nc, c = (int)I.c;
    const int nblk_all = (p + (1 << kAttBlockLog)) >> kAttBlockLog;    // blocks containing positions <= p (the new one included)
    const int my_blocks = (nblk_all > c) ? (nblk_all - c + nc - 1) / nc : 0;
    st.p = p;
    st.nblk = my_blocks > wave ? (my_blocks - wave + kWaves - 1) / kWaves : 0;
    const size_t head_elems = (size_t)P.max_context * D;
    const uint16_t *Kc = P.kv + ((((size_t)I.layer * 2 + 0) * P.max_batch + b) * P.n_kv_heads + g) * head_elems;
    const uint16_t *Vc = P.kv + ((((size_t)I.layer * 2 + 1) * P.max_batch + b) * P.n_kv_heads + g) * head_elems;
    st.kp = (gp)(uintptr_t)Kc + (lane >> 4);
    st.vp = (gp)(uintptr_t)Vc + (lane >> 4);
    if (p > 0) {
#pragma unroll
        for (int s = 0; s < kAttMcDepth; ++s)
            if (s < st.nblk) att_mc_load<D>(I, st, s, s);
    }
}

template <int D>
__device__ __forceinline__ void att_task_mc(const Params &P, const InstrAtt &I, char *lds, Wg &lp, AttStreamMc<D> &as, uint32_t pc)
{
    constexpr int ND = D / 32, NV = D / 16, MS = D + 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = (int)rfl((uint32_t)tid >> 6);
    const int b = (int)I.b, g = (int)I.g;
    if (b >= P.batch) return;
    const int GG = P.n_q_heads / P.n_kv_heads, hb = (int)I.h0, G = (int)I.nh;
    const int p = as.p;
    float *sq = (float *)(lds + lp.xs_off);              // [kMaxGroup][D] rotated, pre-scaled q
    float *snew = sq + kMaxGroup * D;                    // [2][D] new k and v
    char *vt = (char *)(snew + 2 * D) + (size_t)wave * (D * kVtRow);   // this wavefront's transposed V block [D][16 positions]
    float *smerge = (float *)((char *)(snew + 2 * D) + (size_t)kWaves * (D * kVtRow));   // [kWaves][G][MS]
    const bool owner = att_prologue<D>(P, I, lds, lp, p, pc);

    const int col = lane & 15, r = lane >> 4;   // operand / result column; 16-byte slice (operands), row group (results)
    const int h = col >> 1, term = col & 1;     // head of the column inside this task; 0: hi term, 1: lo term
    // B operand of the score products: this column's q term, k = 32 i + 8 r .. + 8
    bf16x8 qop[ND];
#pragma unroll
    for (int i = 0; i < ND; ++i) {
        const f32x4 *qp = (const f32x4 *)(sq + (h < G ? h : 0) * D + 32 * i + 8 * r);
        f32x4 a = qp[0], c4 = qp[1];
        u32x4 pk = {pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w), pack_bf16x2(c4.x, c4.y), pack_bf16x2(c4.z, c4.w)};
        if (term) {
            a.x -= bf_lo(pk.x); a.y -= bf_hi(pk.x); a.z -= bf_lo(pk.y); a.w -= bf_hi(pk.y);
            c4.x -= bf_lo(pk.z); c4.y -= bf_hi(pk.z); c4.z -= bf_lo(pk.w); c4.w -= bf_hi(pk.w);
            pk = u32x4{pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w), pack_bf16x2(c4.x, c4.y), pack_bf16x2(c4.z, c4.w)};
        }
        if (h >= G) pk = u32x4{0u, 0u, 0u, 0u};
        qop[i] = __builtin_bit_cast(bf16x8, pk);
    }

    float M = -INFINITY, lsum = 0.f;
    f32x4 acc[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int nc = (int)I.nc, c = (int)I.c;
    const int jb_new = p >> kAttBlockLog;
    auto swap2 = [](float v) { return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, true)); };
    auto pair = [](float lo, float hi) { return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xffff0000u); };

    auto block = [&](int s, int kk) {
        const int jb = c + (wave + kk * kWaves) * nc;        // block of the cache
        const int t0 = jb << kAttBlockLog;
        u32x4 kr[ND], vr[ND];
#pragma unroll
        for (int i = 0; i < ND; ++i) { kr[i] = as.kbuf[s][i]; vr[i] = as.vbuf[s][i]; }
        if (owner && jb == jb_new && col == (p & 15)) {
            // the new position: its rows come from LDS (bf16-rounded like the rows in the cache); the loads went to row p - 1
#pragma unroll
            for (int i = 0; i < ND; ++i) {
                const float *kn = snew + 32 * i + 8 * r, *vn = snew + D + 32 * i + 8 * r;
                const f32x4 k0 = *(const f32x4 *)kn, k1 = *(const f32x4 *)(kn + 4), v0 = *(const f32x4 *)vn, v1 = *(const f32x4 *)(vn + 4);
                kr[i] = u32x4{pair(k0.x, k0.y), pair(k0.z, k0.w), pair(k1.x, k1.y), pair(k1.z, k1.w)};
                vr[i] = u32x4{pair(v0.x, v0.y), pair(v0.z, v0.w), pair(v1.x, v1.y), pair(v1.z, v1.w)};
            }
        }
        // the V block, transposed, into this wavefront's LDS rows: VT[d][position] (LDS requests of a wavefront are served in
        // order, so these stores cannot overtake the reads of the previous block)
        {
            char *wb = vt + (8 * r) * kVtRow + 2 * col;
#pragma unroll
            for (int i = 0; i < ND; ++i) {
                const uint32_t dw[4] = {vr[i].x, vr[i].y, vr[i].z, vr[i].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    *(uint16_t *)(wb + (32 * i + 2 * q) * kVtRow) = (uint16_t)(dw[q] & 0xffffu);
                    *(uint16_t *)(wb + (32 * i + 2 * q + 1) * kVtRow) = (uint16_t)(dw[q] >> 16);
                }
            }
        }
        // scores of the 16 positions against every column
        f32x4 sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < ND; ++i) sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kr[i]), qop[i], sc, 0, 0, 0);
        float sv[4], bmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float v = sc[j] + swap2(sc[j]);                       // hi + lo column of the head
            sv[j] = (t0 + 4 * r + j <= p) ? v : -INFINITY;              // sc[j]: position t0 + 4 r + j
            bmax = fmaxf(bmax, sv[j]);
        }
        if (__any(bmax > M)) {
            // some column's maximum rises: agree on it across the four row groups, rescale that column's sums
            float mn = fmaxf(M, bmax);
            mn = fmaxf(mn, __shfl_xor(mn, 16, 64));
            mn = fmaxf(mn, __shfl_xor(mn, 32, 64));
            const float rs = safe_exp_diff(M, mn);
            lsum *= rs;
#pragma unroll
            for (int i = 0; i < NV; ++i) acc[i] *= rs;
            M = mn;
        }
        float pr[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) pr[j] = safe_exp_diff(sv[j], M);
        lsum += (pr[0] + pr[1]) + (pr[2] + pr[3]);
        uint32_t p01 = pack_bf16x2(pr[0], pr[1]), p23 = pack_bf16x2(pr[2], pr[3]);
        if (term) {
            p01 = pack_bf16x2(pr[0] - bf_lo(p01), pr[1] - bf_hi(p01));
            p23 = pack_bf16x2(pr[2] - bf_lo(p23), pr[3] - bf_hi(p23));
        }
        typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
        const s16x4 pop = __builtin_bit_cast(s16x4, u32x2v{p01, p23});
        const char *rb = vt + col * kVtRow + 8 * r;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const s16x4 va = *(const s16x4 *)(rb + 16 * i * kVtRow);   // V^T[16 i + lane % 16][4 r .. 4 r + 3]
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, pop, acc[i], 0, 0, 0);
        }
    };

    for (int base = 0; base < as.nblk; base += kAttMcDepth) {
#pragma unroll
        for (int s = 0; s < kAttMcDepth; ++s) {
            if (base + s < as.nblk) {            // (wave-uniform)
                block(s, base + s);
                if (base + s + kAttMcDepth < as.nblk) att_mc_load<D>(I, as, s, base + s + kAttMcDepth);   // (implies p > 0)
            }
        }
    }
    trace_mark(P, pc, 1);

    // ---- this wavefront's state per head: the denominators of the four row groups and the two term columns add up
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += swap2(acc[i][j]);
    if (term == 0 && h < G) {
        float *dst = smerge + ((size_t)wave * G + h) * MS;
#pragma unroll
        for (int i = 0; i < NV; ++i) *(f32x4 *)(dst + 16 * i + 4 * r) = acc[i];      // acc[i][j]: d = 16 i + 4 r + j
        if (r == 0) { dst[D] = M; dst[D + 1] = lsum; }
    }
    wg_sync(lp, lds);
    trace_mark(P, pc, 2);

    // merged max, denominator and per-wavefront weights of every head: thread (head, wavefront), a head's four in one quad
    float *sfac = smerge + (size_t)kWaves * G * MS;     // [G][kWaves] weights, then [G] max, [G] denominators
    static_assert(kWaves == 4, "the merge reduces over quads of lanes");
    if (tid < G * kWaves) {
        const int hh = tid / kWaves, w = tid % kWaves;
        const float *src = smerge + ((size_t)w * G + hh) * MS;
        const float m = src[D], l = src[D + 1];
        float Mx = dpp_max<0xB1>(m);
        Mx = dpp_max<0x4E>(Mx);
        const float f = safe_exp_diff(m, Mx);
        float L = dpp_add<0xB1>(f * l);
        L = dpp_add<0x4E>(L);
        sfac[hh * kWaves + w] = f;
        if (w == 0) { sfac[G * kWaves + hh] = Mx; sfac[G * kWaves + G + hh] = L; }
    }
    wg_sync(lp, lds);
    const ActBuf ab = act_buf(P);
    for (int e = tid; e < G * D / 4; e += kWgThreads) {       // four adjacent outputs per thread
        const int hh = (4 * e) / D, i = (4 * e) % D;
        f32x4 svv[kWaves];
        float fv[kWaves];
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            svv[w] = *(const f32x4 *)(smerge + ((size_t)w * G + hh) * MS + i);
            fv[w] = sfac[hh * kWaves + w];
        }
        f32x4 A = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < kWaves; ++w) A += svv[w] * fv[w];
        // partial layout [b][head][nc][D + kPartStride]
        const uint32_t dst = I.out + (uint32_t)((((size_t)b * P.n_q_heads + (g * GG + hb + hh)) * I.nc + I.c) * (D + kPartStride));
        st_act4(ab, dst + (uint32_t)i, A);
        if (i == 0) {
            float *ml = (float *)(P.scr + P.lay.act) + dst + D;
            st_act(ml, sfac[G * kWaves + hh]);
            st_act(ml + 1, sfac[G * kWaves + G + hh]);
        }
    }
    trace_mark(P, pc, 3);
}

// Combine the nc flash-decode partials of q heads h0 .. h0+nh of sequence b: the partial rows
// are copied to LDS with all their 128-bit loads in flight together, then reduced in fixed order.
__device__ __forceinline__ void comb_task(const Params &P, const InstrAtt &I, char *lds, Wg &lp)
{
    const int b = (int)I.b;
    if (b >= P.batch) return;
    const int D = P.head_dim, nc = (int)I.nc, RS = D + kPartStride;
    const ActBuf ab = act_buf(P);
    float *stage = (float *)(lds + lp.xs_off);
    float *o = (float *)(P.scr + P.lay.act) + I.o_out + (size_t)b * I.o_ld;
    const int lane = threadIdx.x & 63, wave = (int)rfl(threadIdx.x >> 6);
    constexpr int U = 9;   // 128-bit loads in flight per lane: one round trip for 64 partial rows of a 128-wide head
    for (int hh = 0; hh < (int)I.nh; ++hh) {
        const int h = (int)I.h0 + hh;
        const uint32_t src = I.out + (uint32_t)(((size_t)b * P.n_q_heads + h) * nc) * (uint32_t)RS;
        const int nq4 = nc * RS / 4;
        float *wgt = stage + (size_t)nc * RS;                    // [nc] merge weights f_c / L
        if (hh) wg_sync(lp, lds);
        for (int q0 = threadIdx.x; q0 < nq4; q0 += kWgThreads * U) {
            f32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int q = q0 + u * kWgThreads;
                v[u] = ld_act4(ab, q < nq4 ? src + 4u * q : 0xfffffff0u);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int q = q0 + u * kWgThreads;
                if (q < nq4) *(f32x4 *)(stage + 4 * q) = v[u];
            }
        }
        wg_sync(lp, lds);
        if (wave == 0) {
            // merge weights once per chunk (lane c, c + 64, ...), in fixed order
            float M = -INFINITY;
            for (int c = lane; c < nc; c += 64) M = fmaxf(M, stage[c * RS + D]);
            M = wave_max(M);
            float L = 0.f;
            for (int c = lane; c < nc; c += 64) L += stage[c * RS + D + 1] * safe_exp_diff(stage[c * RS + D], M);
            L = wave_sum(L);
            for (int c = lane; c < nc; c += 64) wgt[c] = safe_exp_diff(stage[c * RS + D], M) / L;
        }
        wg_sync(lp, lds);
        for (int i = threadIdx.x; i < D; i += kWgThreads) {
            float A = 0.f;
            int c = 0;
            for (; c + 8 <= nc; c += 8) {      // eight rows' reads in flight, summed in chunk order
                float sv[8], fv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) { sv[u] = stage[(c + u) * RS + i]; fv[u] = wgt[c + u]; }
#pragma unroll
                for (int u = 0; u < 8; ++u) A += sv[u] * fv[u];
            }
            for (; c < nc; ++c) A += stage[c * RS + i] * wgt[c];
            st_act(o + (size_t)h * D + i, A);
        }
    }
}

// Residual sum: this workgroup's slice of the residual rows of every sequence plus the partial rows a K-sliced
// projection left, summed in slice order and stored as the new residual (all loads of an item in flight together).
__device__ __forceinline__ void rsum_task(const Params &P, const Instr &I)
{
    constexpr uint32_t kMaxParts = 8;
    const ActBuf ab = act_buf(P);
    const uint32_t n4 = (I.xs_hi - I.xs_lo) >> 2, np = min(instr_nparts(I), kMaxParts);
    const uint32_t items = (uint32_t)P.batch * n4;
    for (uint32_t it = threadIdx.x; it < items; it += kWgThreads) {
        const uint32_t b = it / n4, off = b * I.in_ld + I.xs_lo + 4u * (it - b * n4);
        f32x4 v = ld_act4(ab, I.in_base + off), pv[kMaxParts];
#pragma unroll
        for (uint32_t s = 0; s < kMaxParts; ++s) pv[s] = ld_act4(ab, s < np ? I.in_parts + s * I.part_stride + off : kNone);
#pragma unroll
        for (uint32_t s = 0; s < kMaxParts; ++s)
            if (s < np) v += pv[s];
        st_act4(ab, I.xs_out + off, v);
    }
}

// Greedy token of sequence b: reduce the (max logit, row) partials the LM-head tasks left, in slot
// order (ties: smaller row, i.e. the first maximum), and hand the row to the caller and to the
// next step of this launch.
__device__ __forceinline__ void argmax_task(const Params &P, const InstrAtt &I, char *lds, Wg &lp)
{
    const int b = (int)I.b, tid = threadIdx.x, lane = tid & 63, wave = (int)rfl((uint32_t)tid >> 6);
    if (b >= P.batch || !P.want_tokens) return;
    const float *part = (const float *)(P.scr + P.lay.act) + I.out;
    float bv = -INFINITY;
    uint32_t bi = 0xffffffffu;
    for (uint32_t s0 = tid; s0 < I.n_slots; s0 += kWgThreads * 4) {
        float v[4], x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t sl = min(s0 + u * kWgThreads, I.n_slots - 1);
            v[u] = ld_act(part + ((size_t)sl * P.max_batch + b) * 2);
            x[u] = ld_act(part + ((size_t)sl * P.max_batch + b) * 2 + 1);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t row = __float_as_uint(x[u]);
            if (s0 + u * kWgThreads < I.n_slots && (v[u] > bv || (v[u] == bv && row < bi))) { bv = v[u]; bi = row; }
        }
    }
    argmax_wave(bv, bi);
    float *sv = (float *)(lds + kLdsMisc + 64);
    uint32_t *si = (uint32_t *)(lds + kLdsMisc + 80);
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    wg_sync(lp, lds);
    if (tid == 0) {
        for (int w = 1; w < kWaves; ++w)
            if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
        if (bi >= (uint32_t)P.vocab) bi = 0;   // no finite logit at all
        typedef __attribute__((address_space(1))) uint32_t *gptr;
        __hip_atomic_store((gptr)(uintptr_t)(lp.tok_out + b), bi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---------------------------------------------------------------- interpreter
__device__ __forceinline__ void fetch_instr(const uint32_t *list, uint32_t pc, uint32_t *slot)
{
    if (threadIdx.x < kInstrDwords) slot[threadIdx.x] = list[(size_t)pc * kInstrDwords + threadIdx.x];
}

// Which GEMV bodies a kernel carries.  A schedule uses one family throughout, so each kernel is
// compiled with only the code it can reach (smaller code, fewer live registers).
enum Path : int {
    kPathValu = 0,    // bf16 weights, VALU dot products (batch 1)
    kPathMfma = 1,    // bf16 weights, matrix cores (any batch)
    kPathW4 = 2,      // 4-bit decoder projections (VALU), bf16 LM head
    kPathAny16 = 3,   // bf16 weights, VALU or matrix cores by the instruction's flag
    kPathW4M = 4,     // 4-bit decoder projections and bf16 LM head, both on the matrix cores (any batch)
};

// Executes one instruction.  `PERSISTENT`: wait on / signal the dependency counters.
template <bool PERSISTENT, bool RING, int PATH>
__device__ __forceinline__ void exec_instr(const Params &P, Wg &lp, char *lds, const Instr &I, uint32_t pc,
                                           bool &dead, uint32_t nxt = 0, uint32_t *nxt_slot = nullptr, bool fill_only = false,
                                           bool one_step = true)
{
    const int tid = threadIdx.x;
    lp.pc = pc;
    uint32_t *sflag = (uint32_t *)(lds + kLdsMisc + 128);
    const uint32_t *counters = (const uint32_t *)(P.scr + P.lay.counters);
    uint64_t t0 = 0, t1 = 0;
    const bool tracing = PERSISTENT && (P.flags & 1u);
    if (tracing && tid == 0) t0 = wall_clock64();

    // Nothing to wait for: the first step of a launch follows the previous launch in stream order,
    // and an arg-max task whose result nobody takes only has to signal.
    // (in a launch of several steps the arg-max tasks always wait: their counter is what orders the steps)
    const bool no_dep = ((I.flags & F_WAIT_PREV) && lp.pos_off == 0) || (I.op == OP_ARGMAX && !P.want_tokens && one_step);
    const bool waiting = PERSISTENT && !dead && !no_dep;
    constexpr bool W4 = PATH == kPathW4 || PATH == kPathW4M;
    uint64_t t2 = 0;

    // The dependency wait of the task; called once, after the task's prefetch has been issued.
    auto await = [&]() {
        if (PERSISTENT) {
            if (tid < 64) {   // the first wave polls
                uint32_t ok = 1, polls = 0;
                if (waiting) {
                    if (I.wait_ctr[0] != kNone)
                        ok = wait_counter(P, counters, I.wait_ctr[0], (lp.epoch - ((I.flags & F_WAIT_PREV) ? 1u : 0u)) * I.wait_cnt[0],
                                          &polls) ? 1u : 0u;
                    if (ok && I.wait_ctr[1] != kNone)
                        ok = wait_counter(P, counters, I.wait_ctr[1], lp.epoch * I.wait_cnt[1], &polls) ? 1u : 0u;
                }
                if (tid == 0) {
                    if (!ok) set_err(P, 0, 1u + pc);
                    sflag[0] = ok;
                    if (I.op == OP_GEMV) {
                        trace_mark(P, pc, 1);
                        if (tracing) ((uint64_t *)(P.ws + P.lay.trace))[((size_t)blockIdx.x * P.max_instr + pc) * 8 + 6] = polls;   // mark 2: polls issued
                    }
                }
            }
            // The next instruction (loaded by the caller before this task began) has certainly arrived
            // by now; parking it in its LDS slot here means nothing waits on memory between the end
            // of this task and the start of the next one.
            if (nxt_slot && tid < kInstrDwords) nxt_slot[tid] = nxt;
            wg_sync(lp, lds);
            if (sflag[0] == 0) dead = true;
        }
        if (tracing && tid == 0) t1 = wall_clock64();
    };

    // Each kind of task is one straight path (prefetch, wait, work), so that the prefetch registers
    // of one kind are not kept alive across the code of another.
    if (fill_only && I.op == OP_GEMV && (I.flags & F_LOGITS)) {
        await();     // a cache fill takes no logits: the LM-head tasks keep their place in the dependency chain, nothing else
    } else if (I.op == OP_GEMV) {
        GemvStream st;
        gemv_issue<RING, W4>(P, I, st, lp.npf);
        if (PERSISTENT) trace_mark(P, pc, 0);
        await();
        if (PATH == kPathMfma || PATH == kPathW4M || (PATH == kPathAny16 && (I.flags & F_MFMA))) {
            if (!(I.flags & F_SKIP_PRO)) gemv_prologue<true>(P, I, lds, lp, P.batch);
            if (tracing && tid == 0) t2 = wall_clock64();
            if (PATH == kPathW4M && (I.flags & F_W4)) gemv_main<true, false, true>(P, I, lds, lp, st, P.batch);
            else gemv_main<true, RING>(P, I, lds, lp, st, P.batch);
        } else {
            if (!(I.flags & F_SKIP_PRO)) gemv_prologue<false>(P, I, lds, lp, 1);
            if (tracing && tid == 0) t2 = wall_clock64();
            if (W4 && (I.flags & F_W4)) gemv_main<false, false, true>(P, I, lds, lp, st, 1);
            else gemv_main<false, RING>(P, I, lds, lp, st, 1);
        }
    } else if (I.op == OP_ATT && (PATH == kPathMfma || PATH == kPathW4M || PATH == kPathAny16) && (I.flags & F_ATT_MC)) {
        const InstrAtt &A = *(const InstrAtt *)&I;
        if (P.head_dim == 128) {
            AttStreamMc<128> as;
            att_issue_mc<128>(P, lp, A, as);
            await();
            att_task_mc<128>(P, A, lds, lp, as, pc);
        } else {
            AttStreamMc<64> as;
            att_issue_mc<64>(P, lp, A, as);
            await();
            att_task_mc<64>(P, A, lds, lp, as, pc);
        }
    } else if (I.op == OP_ATT && PATH != kPathMfma && PATH != kPathW4M) {   // (the matrix-core kernels carry only the form above)
        const InstrAtt &A = *(const InstrAtt *)&I;
        AttStream as;
        if (P.head_dim == 128) {
            att_issue<128>(P, lp, A, as);
            await();
            if (A.nh <= 4) att_task<128, 4>(P, A, lds, lp, as, pc);
            else att_task<128, kMaxGroup>(P, A, lds, lp, as, pc);
        } else {
            att_issue<64>(P, lp, A, as);
            await();
            if (A.nh <= 4) att_task<64, 4>(P, A, lds, lp, as, pc);
            else att_task<64, kMaxGroup>(P, A, lds, lp, as, pc);
        }
    } else {
        await();
        if (I.op == OP_COMB) comb_task(P, *(const InstrAtt *)&I, lds, lp);
        else if (I.op == OP_ARGMAX) argmax_task(P, *(const InstrAtt *)&I, lds, lp);
        else if (I.op == OP_RSUM) rsum_task(P, I);
    }

    if (PERSISTENT && I.sig_ctr != kNone) {
        // each wave drains its write-through stores, the barrier collects all waves, then one
        // thread publishes the task with the counter increment
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        wg_sync(lp, lds);
        if (tid == 0)
            __hip_atomic_fetch_add((uint32_t *)sub_counter(P, counters, I.sig_ctr, blockIdx.x & (kCounterSubs - 1u)), 1u,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tracing && tid == 0) {
        uint64_t *r = (uint64_t *)(P.ws + P.lay.trace) + ((size_t)blockIdx.x * P.max_instr + pc) * 8;
        r[0] = t0; r[1] = t1; r[2] = t2 ? t2 : t1; r[3] = wall_clock64();
    }
}

__device__ __forceinline__ void read_instr(const uint32_t *slot, Instr &I)
{
    uint32_t *dst = (uint32_t *)&I;
#pragma unroll
    for (int j = 0; j < kInstrDwords; ++j) dst[j] = rfl(slot[j]);
}

__device__ __forceinline__ Wg make_wg(const Params &P, const LdsPlan &p, char *lds, bool ring, int npf = kPrefetch)
{
    typedef __attribute__((address_space(3))) char *lptr;
    Wg wg;
    wg.red_bytes = p.red_bytes; wg.xs_off = p.xs_off;
    wg.ring = ring; wg.npf = npf;
    wg.wave = rfl(threadIdx.x >> 6);
    wg.nst = p.ring_slots / (kWaves * kStagePages);
    wg.ring_off = p.ring_off + wg.wave * wg.nst * kStagePages * kChunkBytes;
    wg.ring_lds = (uint32_t)(uintptr_t)(lptr)lds + wg.ring_off;
    wg.head = wg.tail = 0; wg.hst = wg.tst = 0;
    wg.pf_ptr = wg.pf_begin = (cptr)(uintptr_t)((const uint32_t *)(P.ws + P.lay.stream) + (size_t)blockIdx.x * P.max_instr * 2);
    wg.pf_left = P.max_instr;
    wg.pf_steps = P.n_steps > 0 ? (uint32_t)P.n_steps - 1u : 0u;
    wg.epoch = P.epoch; wg.pos_off = 0;
    if (P.epoch_ptr) {
        typedef const __attribute__((address_space(1))) uint32_t *gptr;
        wg.epoch = rfl(__hip_atomic_load((gptr)(uintptr_t)P.epoch_ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    } wg.tok_src = P.tokens; wg.tok_out = P.next_tokens; wg.logits = P.logits;
    wg.pf_src = nullptr; wg.pf_rem = 0; wg.pf_live = wg.ring && wg.nst > 0;
    return wg;
}

// Persistent walk of this workgroup's whole list; the next instruction is fetched while the
// current one runs.
template <bool RING, bool MULTI, int PATH>
__device__ __forceinline__ void run_persistent(const Params &P, const LdsPlan plan)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    Wg lp = make_wg(P, plan, lds, RING);
    if (RING)   // fill the ring with the first stages of this wave's stream
        for (uint32_t i = 0; i < lp.nst; ++i) ring_fill_stage(P, lp);
    const uint32_t *list = (const uint32_t *)(P.ws + P.lay.instr) + (size_t)blockIdx.x * P.max_instr * kInstrDwords;
    uint32_t *sinstr = (uint32_t *)(lds + kLdsInstr);   // two slots of 32 dwords
    bool dead = false;   // a wait timed out: stop waiting, keep walking so the grid drains
    // A launch walks the list once per decode step.  Step s decodes the greedy tokens of step s-1 at
    // the caller's positions + s; its tasks are ordered after step s-1 by the arg-max counter.
    const int n_steps = MULTI ? P.n_steps : 1;   // the single-step kernel keeps the step context constant
    const uint32_t epoch0 = lp.epoch;            // (the launch's argument, or the number kept in device memory)
    for (int step = 0; step < n_steps; ++step) {
        lp.epoch = epoch0 + (uint32_t)step;
        lp.pos_off = step;
        lp.tok_src = step ? P.next_tokens + (size_t)(step - 1) * P.batch : P.tokens;
        if (MULTI && P.forced_tokens) lp.tok_src = P.forced_tokens + (size_t)step * P.batch;
        lp.tok_out = P.next_tokens + (size_t)step * P.batch;
        wg_sync(lp, lds);   // the previous walk's last instruction has been read by every wave
        fetch_instr(list, 0, sinstr);
        for (uint32_t pc = 0; pc < P.max_instr; ++pc) {
            wg_sync(lp, lds);
            Instr I;
            read_instr(sinstr + (pc & 1u) * kInstrDwords, I);
            if (I.op == OP_END) break;
            uint32_t nxt = 0;
            const bool more = pc + 1 < P.max_instr;
            if (more && threadIdx.x < kInstrDwords) nxt = list[(size_t)(pc + 1) * kInstrDwords + threadIdx.x];
            if (RING) pin_uniform(lp);
            exec_instr<true, RING, PATH>(P, lp, lds, I, pc, dead, nxt, more ? sinstr + ((pc + 1) & 1u) * kInstrDwords : nullptr,
                                         MULTI && P.forced_tokens != nullptr,
                                         // (a launch of one step.  The single-step vector kernel tests the argument although it
                                         // is 1 there by construction: with the constant it measured 2 % slower -- these kernels
                                         // spill scalar registers, and where the spills land moves with details like this one)
                                         (PATH == kPathValu && !MULTI) ? P.n_steps <= 1 : (!MULTI || n_steps <= 1));
        }
    }
    // no DMA load may still be writing LDS when the workgroup retires
    if (RING) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// One operator instance: the instructions of this workgroup whose ref_seq matches (they are
// adjacent in the list), found with one parallel scan.
template <int PATH>
__device__ __forceinline__ void run_one_op(const Params &P, const LdsPlan plan)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    Wg lp = make_wg(P, plan, lds, false);
    const uint32_t *list = (const uint32_t *)(P.ws + P.lay.instr) + (size_t)blockIdx.x * P.max_instr * kInstrDwords;
    uint32_t *sinstr = (uint32_t *)(lds + kLdsInstr);
    uint32_t *srange = (uint32_t *)(lds + kLdsMisc + 160);   // [0] first match, [1] match count
    if (threadIdx.x == 0) { srange[0] = 0xffffffffu; srange[1] = 0u; }
    wg_sync(lp, lds);
    for (uint32_t i = threadIdx.x; i < P.max_instr; i += kWgThreads) {
        uint32_t op = list[(size_t)i * kInstrDwords], seq = list[(size_t)i * kInstrDwords + 2];
        if (op != OP_END && seq == P.only_seq) { atomicMin(srange, i); atomicAdd(srange + 1, 1u); }
    }
    wg_sync(lp, lds);
    const uint32_t first = srange[0], n = srange[1];
    bool dead = false;
    for (uint32_t pc = first; pc < first + n && n; ++pc) {
        wg_sync(lp, lds);
        fetch_instr(list, pc, sinstr);
        wg_sync(lp, lds);
        Instr I;
        read_instr(sinstr, I);
        exec_instr<false, false, PATH>(P, lp, lds, I, pc, dead);
    }
}

}  // namespace mk

#define MK_KERNEL(name, body) \
    extern "C" __global__ void __launch_bounds__(mk::kWgThreads) name(const mk::Params P, const mk::LdsPlan lp) { body; }

// One walk of the lists (one decode step) / the walk repeated once per decode step of the launch
// (greedy token feedback on the device) / one operator instance per launch, for each GEMV family.
// The families are kept apart so that the batch-1 bf16 kernels carry none of the matrix-core or W4 code.
MK_KERNEL(mk_megakernel, (mk::run_persistent<false, false, mk::kPathValu>(P, lp)))
MK_KERNEL(mk_megakernel_steps, (mk::run_persistent<false, true, mk::kPathValu>(P, lp)))
MK_KERNEL(mk_op_kernel, (mk::run_one_op<mk::kPathValu>(P, lp)))
MK_KERNEL(mk_megakernel_mfma, (mk::run_persistent<false, false, mk::kPathMfma>(P, lp)))
MK_KERNEL(mk_megakernel_steps_mfma, (mk::run_persistent<false, true, mk::kPathMfma>(P, lp)))
MK_KERNEL(mk_op_kernel_mfma, (mk::run_one_op<mk::kPathMfma>(P, lp)))
MK_KERNEL(mk_megakernel_w4, (mk::run_persistent<false, false, mk::kPathW4>(P, lp)))
MK_KERNEL(mk_megakernel_steps_w4, (mk::run_persistent<false, true, mk::kPathW4>(P, lp)))
MK_KERNEL(mk_op_kernel_w4, (mk::run_one_op<mk::kPathW4>(P, lp)))
MK_KERNEL(mk_megakernel_w4m, (mk::run_persistent<false, false, mk::kPathW4M>(P, lp)))
MK_KERNEL(mk_megakernel_steps_w4m, (mk::run_persistent<false, true, mk::kPathW4M>(P, lp)))
MK_KERNEL(mk_op_kernel_w4m, (mk::run_one_op<mk::kPathW4M>(P, lp)))
// Any step count, with the per-wave LDS page ring carrying the weight stream (bf16, either GEMV body).
MK_KERNEL(mk_megakernel_ring, (mk::run_persistent<true, true, mk::kPathAny16>(P, lp)))

// Offline weight reorder: row-major bf16 [n_rows][n_cols] -> tile-major chunks of R = 1 << rlog rows.
// Source row i lands in row group g0 + i / rpu at row r_off + i % rpu of the group (rpu = R and
// r_off = 0 for a plain matrix; rpu = R/2 with r_off 0 / R/2 interleaves the gate and up matrices).
// Chunk (group, kb) holds lane-major 16 B: lane = ksub * R + r -> W[row][kb * 512/R + ksub*8 + 0..7].
// Lanes whose r lies outside [r_off, r_off + rpu) belong to the other matrix and are left alone;
// rows and columns beyond the source are written as zeros.  `ord` says where chunk (group, kb) is stored (chunk_slot).
extern "C" __global__ void mk_repack_kernel(const uint16_t *src, int n_rows, int n_cols, mk::u32x4 *dst, uint32_t kbt,
                                            uint32_t rlog, uint32_t rpu, uint32_t r_off, uint32_t g0, uint32_t n_groups,
                                            mk::ChunkOrder ord)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)n_groups * kbt * 64;
    if (gid >= total) return;
    const uint32_t R = 1u << rlog, ck = 512u >> rlog;
    uint32_t lane = (uint32_t)(gid & 63);
    size_t c = gid >> 6;
    uint32_t kb = (uint32_t)(c % kbt), grp = (uint32_t)(c / kbt);
    uint32_t r = lane & (R - 1), ksub = lane >> rlog;
    if (r < r_off || r >= r_off + rpu) return;
    long row = (long)grp * rpu + (r - r_off);
    int k0 = (int)(kb * ck + ksub * 8);
    uint16_t e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int k = k0 + j;
        e[j] = (row < n_rows && k < n_cols) ? src[(size_t)row * n_cols + k] : (uint16_t)0;
    }
    mk::u32x4 v;
    v.x = e[0] | ((uint32_t)e[1] << 16); v.y = e[2] | ((uint32_t)e[3] << 16);
    v.z = e[4] | ((uint32_t)e[5] << 16); v.w = e[6] | ((uint32_t)e[7] << 16);
    dst[(size_t)mk::chunk_slot(ord.sm != 0, g0 + grp, kb, ord.S, ord.groups, kbt, ord.nkb) * 64 + lane] = v;
}

// Offline reorder of a W4 matrix: codes row-major uint8 [n_rows][n_cols / 2] (even k in the low nibble)
// -> chunks of R rows x 2048/R k; lane = ksub * R + r takes the 16 bytes holding k0 + 32 ksub .. + 32 of
// its row.  Same row-group placement rules as mk_repack_kernel; rows and columns beyond the source are
// code 8 (weight zero).
// With `mfma` (16 rows per chunk) the codes are laid out for the matrix cores instead: dword i of lane ksub * 16 + r
// holds the 8 codes of k0 + 32 i + 8 ksub .. + 8, nibble p standing for offset 2 (p % 4) + p / 4 inside those 8.
extern "C" __global__ void mk_repack_w4_kernel(const uint8_t *src, int n_rows, int n_cols, mk::u32x4 *dst, uint32_t kbt,
                                               uint32_t rlog, uint32_t rpu, uint32_t r_off, uint32_t g0, uint32_t n_groups,
                                               uint32_t mfma, mk::ChunkOrder ord)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)n_groups * kbt * 64;
    if (gid >= total) return;
    const uint32_t R = 1u << rlog, ck = 2048u >> rlog;
    uint32_t lane = (uint32_t)(gid & 63);
    size_t c = gid >> 6;
    uint32_t kb = (uint32_t)(c % kbt), grp = (uint32_t)(c / kbt);
    uint32_t r = lane & (R - 1), ksub = lane >> rlog;
    if (r < r_off || r >= r_off + rpu) return;
    long row = (long)grp * rpu + (r - r_off);
    const int k0 = (int)(kb * ck + ksub * 32);
    uint32_t d[4];
    if (mfma) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t v = 0;
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int k = (int)(kb * ck) + 32 * i + 8 * (int)ksub + 2 * (p % 4) + p / 4;
                uint32_t code = 8u;                                  // absent rows / columns: weight zero
                if (row < n_rows && k < n_cols) {
                    const uint32_t byte = src[(size_t)row * (n_cols / 2) + k / 2];
                    code = (k & 1) ? (byte >> 4) : (byte & 15u);
                }
                v |= code << (4 * p);
            }
            d[i] = v;
        }
        mk::u32x4 v4 = {d[0], d[1], d[2], d[3]};
        dst[(size_t)mk::chunk_slot(ord.sm != 0, g0 + grp, kb, ord.S, ord.groups, kbt, ord.nkb) * 64 + lane] = v4;
        return;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t v = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int k = k0 + 8 * i + 2 * b;   // byte b of dword i: codes of k and k + 1 (n_cols is even)
            const uint32_t byte = (row < n_rows && k < n_cols) ? src[(size_t)row * (n_cols / 2) + k / 2] : 0x88u;
            v |= byte << (8 * b);
        }
        d[i] = v;
    }
    mk::u32x4 v4 = {d[0], d[1], d[2], d[3]};
    dst[(size_t)mk::chunk_slot(ord.sm != 0, g0 + grp, kb, ord.S, ord.groups, kbt, ord.nkb) * 64 + lane] = v4;
}

// The scales that go with it: src bf16 [n_rows][n_cols / group] -> per chunk 2048/group values, index
// g * R + r for group g of the chunk's k range and row r of the chunk; absent rows / groups get 0.
extern "C" __global__ void mk_repack_scales_kernel(const uint16_t *src, int n_rows, int n_cols, uint16_t *dst, uint32_t kbt,
                                                   uint32_t rlog, uint32_t rpu, uint32_t r_off, uint32_t g0,
                                                   uint32_t n_groups, uint32_t group, mk::ChunkOrder ord)
{
    const uint32_t R = 1u << rlog, ck = 2048u >> rlog, spc = 2048u / group;
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)n_groups * kbt * spc;
    if (gid >= total) return;
    uint32_t si = (uint32_t)(gid % spc);
    size_t c = gid / spc;
    uint32_t kb = (uint32_t)(c % kbt), grp = (uint32_t)(c / kbt);
    uint32_t r = si & (R - 1), g = si >> rlog;
    if (r < r_off || r >= r_off + rpu) return;
    long row = (long)grp * rpu + (r - r_off);
    const uint32_t kg = (kb * ck) / group + g;       // group index along K
    const uint32_t n_kg = (uint32_t)n_cols / group;
    dst[(size_t)mk::chunk_slot(ord.sm != 0, g0 + grp, kb, ord.S, ord.groups, kbt, ord.nkb) * spc + si] = (row < n_rows && kg < n_kg) ? src[(size_t)row * n_kg + kg] : (uint16_t)0;
}

extern "C" __global__ void mk_copy_u16_kernel(const uint16_t *src, uint16_t *dst, size_t n)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < n) dst[gid] = src[gid];
}

// Opens a step on the static scratch array (one workgroup): advances the step number kept in device memory and, when
// asked to or when the number comes near the range where (step number x signals) would wrap, zeroes the dependency
// counters and starts again from 1.  Being a kernel, it does the right thing at every replay of a recorded graph.
extern "C" __global__ void __launch_bounds__(1024) mk_static_begin_kernel(uint32_t *epoch, uint32_t *counters, size_t n_dwords, uint32_t reset)
{
    __shared__ uint32_t cur;
    if (threadIdx.x == 0) cur = *epoch;
    __syncthreads();
    const bool zero = reset != 0u || cur >= 0x00800000u;
    if (zero)
        for (size_t i = threadIdx.x; i < n_dwords; i += blockDim.x) counters[i] = 0u;
    __syncthreads();
    if (threadIdx.x == 0) *epoch = zero ? 1u : cur + 1u;
}

extern "C" __global__ void mk_fill_u32_kernel(uint32_t *dst, uint32_t v, size_t n)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < n) dst[gid] = v;
}


// Streaming-read ceiling of the device: a persistent grid (one workgroup per CU) in which every workgroup reads
// its contiguous share of a buffer with the load form of the GEMV weight stream (128-bit nontemporal loads, 16 in
// flight per lane), and nothing else.  What this kernel reaches is the bandwidth a weight stream can reach at all.
extern "C" __global__ void __launch_bounds__(256) mk_stream_read_kernel(const mk::u32x4 *src, uint32_t chunks_per_wg, uint32_t *sink)
{
    constexpr int kDepth = 16;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const mk::u32x4 *base = src + (size_t)blockIdx.x * chunks_per_wg * 64 + lane;
    const uint32_t total = chunks_per_wg, last = total ? total - 1 : 0;
    mk::u32x4 acc = {0u, 0u, 0u, 0u};
    mk::u32x4 buf[kDepth];
#pragma unroll
    for (int j = 0; j < kDepth; ++j) buf[j] = __builtin_nontemporal_load(base + (size_t)min(wave + 4u * j, last) * 64);
    for (uint32_t b = 0; b < total; b += 4 * kDepth) {
#pragma unroll
        for (int j = 0; j < kDepth; ++j) {
            const uint32_t idx = b + 4u * j + wave;
            if (idx < total) acc ^= buf[j];
            buf[j] = __builtin_nontemporal_load(base + (size_t)min(idx + 4u * kDepth, last) * 64);
        }
    }
    // the loads must not be optimised away; the condition does not hold for any real buffer content
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x5bd1e995u && sink) sink[0] = acc.x;
}
