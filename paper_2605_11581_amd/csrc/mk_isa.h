// Instruction format, workspace layout and kernel parameters shared by the
// host scheduler and the device interpreter.  Plain C++ PODs, no HIP types.
//
// The static schedule (paper Sec. 4.2.2 Step 4, "execution-path
// solidification") is one array of fixed-size instructions per workgroup.
// Every decision -- which tiles a workgroup computes, in which order, which
// dependency counters it waits on and signals, which LDS pages its weight
// stream lands in -- is a constant of this list; the kernel only walks it.
#pragma once
#include <stdint.h>

#ifndef __HIPCC__
#define __host__
#define __device__
#endif

namespace mk {

constexpr int kWgThreads = 256;        // 4 wavefronts of 64
constexpr int kWaves = kWgThreads / 64;
constexpr int kChunkBytes = 1024;      // one wavefront-wide 128-bit load: 16 rows x 32 k of bf16
constexpr int kInstrDwords = 32;
constexpr uint32_t kNone = 0xffffffffu;
constexpr int kMaxBatch = 16;         // sequences per step: 8 fill the 16 columns of one matrix-core instruction (two bf16
                                       // terms each), 9..16 take a second instruction per weight chunk
constexpr int kActTerms = 2;           // bf16 terms (hi + lo) of an fp32 activation on the matrix-core path
constexpr int kMaxGroup = 8;           // q heads per kv head
constexpr int kCounterStride = 32;     // dwords between sub-counters (one 128-byte line each)
constexpr int kCounterSubs = 16;       // sub-counters per dependency counter (a power of two, at most 16: one poll reads them
                                       // with the first 16 lanes); measured best of 1..64 on MI355X
constexpr int kCounterDwords = kCounterStride * kCounterSubs;   // dwords of the counter region per dependency counter
constexpr int kPrefetch = 6;           // 128-bit bf16 weight loads a lane keeps in flight (direct-load path): 24 KB per
                                       // workgroup; measured best of 4..32 on every shape (deeper bursts delay the
                                       // dependency polls and activation loads queued behind them)

// LDS map of a workgroup:
//   [0, 256)    current instruction
//   [256, 512)  block-reduction scratch, flags
//   [512, ...)  cross-wave partial sums (red), then the staged input vector / attention scratch (xs),
//               then (1 KB aligned) the weight-page ring: ring_slots / 4 pages of 1 KB per wavefront
constexpr int kLdsInstr = 0;
constexpr int kLdsMisc = 256;
constexpr int kLdsRed = 512;

enum Op : uint32_t { OP_END = 0, OP_GEMV = 1, OP_ATT = 2, OP_COMB = 3, OP_ARGMAX = 4, OP_RSUM = 5 };

// stage of an operator instance inside a layer; ref_seq = layer * 8 + stage
enum Stage : uint32_t { ST_QKV = 0, ST_ATT = 1, ST_COMB = 2, ST_O = 3, ST_GU = 4, ST_DOWN = 5, ST_HEAD = 6, ST_ARGMAX = 7,
                        ST_RSUM = 6 };   // (inside a layer; ST_HEAD and ST_ARGMAX only exist behind the last one)

// The down projection's K slices leave S partial rows per sequence, which every task of the next operator would read
// whole.  From about 64 K floats of partial rows on (a level costs about 3.5 us, the re-reading about 0.07 us per thousand
// floats and workgroup) one extra level in which each workgroup sums a slice of the rows once is cheaper.
__host__ __device__ inline bool wants_residual_sum(int s_down, int max_batch, int hidden)
{
    return s_down > 1 && (long)s_down * max_batch * hidden >= 65536;
}

enum Pro : uint32_t {
    PRO_EMBED_NORM = 0,  // x = embedding row; store slice; RMSNorm
    PRO_RESID_NORM = 1,  // x = base + sum(partials); store slice; RMSNorm
    PRO_PLAIN = 2,       // x[k] = sum(partials)[k] over the unit's k range
    PRO_SILU = 3,        // x[k] = silu(sum gate partials[k]) * sum up partials[k]
    PRO_COMBINE = 4      // x = flash-decode combine of the n_parts attention partials of the heads that cover the
                         // unit's k range (the O projection reading the attention partials directly);
                         // in_base = byte offset, inside the staged-input area, of the partial-row staging
};

enum Flags : uint32_t {
    F_SKIP_PRO = 1u,    // LDS already holds this task's input vector (same operator, previous task)
    F_MFMA = 2u,        // matrix-core GEMV/thin GEMM instead of VALU FMA
    F_LOGITS = 4u,      // output goes to the caller's logits buffer
    F_ADD_RESID = 8u,   // epilogue adds the residual row (needs S == 1): out = resid + W x
    F_SILU_EPI = 16u,   // epilogue of the fused gate/up matrix (needs S == 1): out = silu(gate) * up
    F_ARGMAX = 32u,     // LM-head task: also leave (max logit, its row) per sequence in partial slot `spare`
    F_WAIT_PREV = 64u,  // wait_ctr[0] is awaited at the PREVIOUS step's target: the first tasks of a step wait
                        // for the greedy token (and with it for every task) of the step before
    F_W4 = 128u,        // the matrix is stored as 4-bit codes: a chunk holds four times the k of a bf16 chunk
    F_SLICE_MAJOR = 256u, // units (and the matrix's chunks) are numbered K slice first: see unit_place()
    F_ATT_MC = 512u      // attention task: scores and weighted values on the matrix cores (blocks of 16 positions per wavefront)
};

// Weight chunk geometry.  A chunk is one wavefront-wide 128-bit load (1 KB): R rows x (512 / R)
// consecutive k of bf16, lane = ksub * R + r holding W[row0 + r][k0 + 8 ksub .. + 8].  R is a
// per-matrix tiling parameter (16 for the matrix-core path); rlog = log2 R.
__host__ __device__ inline uint32_t chunk_k(uint32_t rlog) { return 512u >> rlog; }
// W4 chunk: R rows x (2048 / R) consecutive k of 4-bit codes, lane = ksub * R + r holding the 32 codes
// W[row0 + r][k0 + 32 ksub .. + 32] (code of k in bits 4 (k mod 8) of dword (k / 8) mod 4).  Every chunk
// has 2048 / group scales (bf16), index (32 ksub / group) * R + r, in a parallel array.
__host__ __device__ inline uint32_t chunk_k_w4(uint32_t rlog) { return 2048u >> rlog; }

// OP_RSUM uses the GEMV view: out[b][lo .. hi) = base[b][lo .. hi) + sum of the n_parts partial rows (in slice order), with
// in_base, in_parts, part_stride, in_ld, cfg (n_parts), xs_lo / xs_hi = [lo, hi) (multiples of 4) and xs_out = out.
struct Instr {                 // 32 dwords
    uint32_t op;               // 0
    uint32_t flags;            // 1
    uint32_t ref_seq;          // 2  topological rank of the operator instance
    uint32_t layer;            // 3
    uint32_t wait_ctr[2];      // 4,5   counter index or kNone
    uint32_t wait_cnt[2];      // 6,7   signals per step the counter receives
    uint32_t sig_ctr;          // 8     counter to signal once the outputs are stored (kNone: none)
    // ---- GEMV: units u0 .. u0+nu of a matrix; unit u = (row group u / S of R rows, K split u % S), or with
    //      F_SLICE_MAJOR (K split u / groups, row group u % groups)
    uint32_t w_chunk;          // 9   first 1 KB chunk of the matrix inside the weight region
    uint32_t kbt;              // 10  chunks per row group (whole K)
    uint32_t nkb;              // 11  chunks per unit (last split of a row group may be shorter)
    uint32_t S;                // 12  K splits per row group
    uint32_t u0;               // 13
    uint32_t nu;               // 14
    uint32_t n_rows;           // 15  valid output rows of the matrix
    uint32_t cfg;              // 16  pro [0:3] | rlog [4:7] | producer rlog (PRO_SILU) [8:11] | n_parts [16:23]
    uint32_t in_base;          // 17  float offset of the residual base (norm prologues)
    uint32_t in_parts;         // 18  float offset of partial 0 / of the plain input vector
    uint32_t resid;            // 19  F_ADD_RESID: float offset of the residual rows added in the epilogue
    uint32_t part_stride;      // 20  floats between partials
    uint32_t in_ld;            // 21  floats between sequences (batch rows) of the input
    uint32_t xs_lo, xs_hi;     // 22,23 norm prologues: slice of the new residual this task stores;
                               //       plain prologues: first staged chunk and number of staged chunks
    uint32_t xs_out;           // 24  float offset of the residual store buffer
    uint32_t gain;             // 25  bf16 element offset of the norm gain in the vector region
    uint32_t out;              // 26  float offset of output partial 0
    uint32_t out_split_stride; // 27  floats between output partials
    uint32_t out_ld;           // 28  floats between sequences of the output
    uint32_t bias;             // 29  bf16 element offset of the bias or kNone
    uint32_t k_len;            // 30  true K (input elements beyond it are zero)
    uint32_t spare;            // 31  F_ARGMAX: slot of this task in the arg-max partial buffer
};
__host__ __device__ inline uint32_t instr_pro(const Instr &I) { return I.cfg & 15u; }
__host__ __device__ inline uint32_t instr_ck(const Instr &I) { return ((I.flags & F_W4) ? 2048u : 512u) >> ((I.cfg >> 4) & 15u); }
__host__ __device__ inline uint32_t instr_rlog(const Instr &I) { return (I.cfg >> 4) & 15u; }
__host__ __device__ inline uint32_t instr_prod_rlog(const Instr &I) { return (I.cfg >> 8) & 15u; }
__host__ __device__ inline uint32_t instr_nparts(const Instr &I) { return (I.cfg >> 16) & 255u; }
__host__ __device__ inline uint32_t instr_groups(const Instr &I) { return (I.n_rows + (1u << instr_rlog(I)) - 1u) >> instr_rlog(I); }

// Unit numbering and chunk order of a matrix cut into S K slices of nkb chunks (the last slice may be shorter) over
// `groups` row groups of kbt chunks each.  Row-group-major (sm = false): unit u = rg * S + s, the chunks of a row group
// are contiguous along K.  Slice-major (sm = true): unit u = s * groups + rg, and the chunks of a slice come first for
// every row group: a run of consecutive units then shares its K range (one staged input slice) AND is one contiguous
// byte range of weights.
__host__ __device__ inline uint32_t slice_chunks(uint32_t s, uint32_t S, uint32_t nkb, uint32_t kbt)
{
    return s + 1u == S ? kbt - s * nkb : nkb;
}
__host__ __device__ inline void unit_place(bool sm, uint32_t u, uint32_t S, uint32_t groups, uint32_t &rg, uint32_t &s)
{
    if (sm) { s = u / groups; rg = u - s * groups; }
    else    { rg = u / S; s = u - rg * S; }
}
// first chunk of unit u, relative to the matrix (u may be one past the last unit)
__host__ __device__ inline uint32_t unit_chunk0(bool sm, uint32_t u, uint32_t S, uint32_t groups, uint32_t kbt, uint32_t nkb)
{
    uint32_t rg, s;
    unit_place(sm, u, S, groups, rg, s);
    if (!sm) return rg * kbt + s * nkb;
    if (s >= S) return groups * kbt;
    return groups * s * nkb + rg * slice_chunks(s, S, nkb, kbt);
}
// where chunk kb of row group grp is stored, relative to the matrix
__host__ __device__ inline uint32_t chunk_slot(bool sm, uint32_t grp, uint32_t kb, uint32_t S, uint32_t groups, uint32_t kbt,
                                               uint32_t nkb)
{
    if (!sm) return grp * kbt + kb;
    uint32_t s = kb / nkb;
    if (s >= S) s = S - 1u;
    return groups * s * nkb + grp * slice_chunks(s, S, nkb, kbt) + (kb - s * nkb);
}
struct ChunkOrder { uint32_t S, nkb, groups, sm; };   // how the offline reorder numbers the chunks of one matrix
__host__ __device__ inline uint32_t make_cfg(uint32_t pro, uint32_t rlog, uint32_t prod_rlog, uint32_t n_parts)
{
    return pro | (rlog << 4) | (prod_rlog << 8) | (n_parts << 16);
}

// ATT / COMB view of the same 32 dwords (fields 0..8 identical).
struct InstrAtt {
    uint32_t op, flags, ref_seq, layer, wait_ctr[2], wait_cnt[2], sig_ctr;
    uint32_t b;                // 9   sequence
    uint32_t g;                // 10  kv head
    uint32_t c;                // 11  chunk task index within (b, g)
    uint32_t nc;               // 12  chunk tasks per (b, g)
    uint32_t bs;               // 13  positions per block (blocks c, c+nc, ... belong to task c)
    uint32_t in_parts;         // 14  float offset of QKV partial 0
    uint32_t n_parts;          // 15
    uint32_t part_stride;      // 16
    uint32_t in_ld;            // 17  floats between sequences in the QKV buffer
    uint32_t qn_gain, kn_gain; // 18,19 bf16 element offsets (qk_norm) or kNone
    uint32_t out;              // 20  float offset of the partial buffer [b][head][nc][d+2]
    uint32_t h0, nh;           // 21,22 COMB: first q head and number of q heads to combine
    uint32_t o_out;            // 23  COMB: float offset of o[b][nq*d]
    uint32_t o_ld;             // 24
    uint32_t n_slots;          // 25  ARGMAX: partial slots to reduce (one per LM-head task)
    uint32_t pad[6];
};
static_assert(sizeof(Instr) == kInstrDwords * 4, "instruction size");
static_assert(sizeof(InstrAtt) == kInstrDwords * 4, "instruction size");

// Byte offsets into the caller-provided workspace.
struct Layout {
    uint64_t weights;    // repacked matrices, 1 KB chunks
    uint64_t wscale;     // W4 only: bf16 scales, 2048 / group per chunk, for the chunks of the decoder layers
    uint64_t vecs;       // bf16 vectors: norm gains, biases
    uint64_t rope;       // float [max_context][head_dim/2][2] (cos, sin)
    uint64_t act;        // fp32 activations, partial sums, attention partials
    uint64_t counters;   // uint32, one per 128-byte line
    uint64_t instr;      // Instr[n_wg][max_instr]
    uint64_t err;        // uint32[8] sticky error flags
    uint64_t trace;      // uint64[n_wg][max_instr][8]: task begin, dependencies met, prologue done, end, 4 task-internal marks
    uint64_t tokens;     // int32[max_batch]: greedy token of the latest step (single-step entry point)
    uint64_t stream;     // uint32[n_wg][max_instr][2]: weight stream of a workgroup, one (first chunk, chunk count) per GEMV
                         // task in list order, closed by (kNone, kNone); derived from the instruction lists at bind time
    uint64_t total;
};

struct Params {
    char *ws;             // the bound workspace: weights, vectors, RoPE table, instruction lists, trace, stream table
    char *scr;            // base of the scratch regions (lay.act, lay.counters, lay.err, lay.tokens are offsets from it):
                          // the workspace itself, or the library's static device array (allocation-free entry point)
    Layout lay;
    const int32_t *tokens;
    const int32_t *positions;
    uint16_t *kv;
    float *logits;
    int32_t *next_tokens;   // [n_steps][batch] greedy tokens, written by the arg-max task of every step
    int32_t n_steps;        // decode steps walked by this launch (token of step s+1 = arg-max of step s)
    int32_t want_tokens;    // 0: the caller takes logits only, the arg-max work is skipped (its tasks still signal)
    const int32_t *forced_tokens;   // cache fill: [n_steps][batch] tokens every step decodes (no feedback); the LM head is
                                    // skipped (its tasks only wait and signal), nothing is written to `logits`
    uint32_t amax;          // float offset of the arg-max partials [slot][max_batch][2] in the activation region
    int32_t batch, max_batch, max_context;
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, inter_pad, vocab;
    int32_t qk_norm;
    float rms_eps;
    uint32_t epoch;       // step number since the counters were last zeroed (>= 1)
    const uint32_t *epoch_ptr;   // non-null: the step number is read from device memory instead (a launch recorded into a graph
                                 // then finds the right number at every replay)
    uint32_t spin_limit;
    uint32_t max_instr;
    uint32_t flags;
    uint32_t embed_chunk; // first chunk of the (repacked) embedding matrix
    uint32_t embed_kbt, embed_rlog;
    uint32_t only_seq;    // per-operator launches: run only instructions with this ref_seq (kNone: all)
    uint32_t act_bytes;   // size of the activation region (buffer-descriptor bound)
    uint32_t w4_group;    // W4: group size along K (32, 64 or 128); 0: bf16 weights
};

}  // namespace mk
