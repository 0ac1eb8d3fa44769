// Host-side schedule object and the offline synthesis entry points
// (paper Sec. 3 Phase I; Sec. 4.1.1; Sec. 4.2.2 Steps 1-4).  No HIP types.
#pragma once
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/mk.h"
#include "mk_isa.h"

namespace mk {

struct Dims {
    int L, H, nq, nkv, d, I, V, Bm, Tm, G;
    int qd, kvd, nqkv;       // fused QKV rows
    int w4, group;           // 1: the decoder projections are 4-bit codes with one scale per `group` k
};

struct Tiling {              // the searched parameters (Sec. 4.2.2 Step 3, "tiling parameter space")
    int s_qkv, s_o, s_gu, s_d;   // K splits
    int r_qkv, r_o, r_gu, r_d, r_head;   // log2 of the rows per weight chunk, per matrix
    int nc;                      // attention chunk tasks per (sequence, kv head)
    int bs;                      // positions per attention block
    int mfma;                    // 0 VALU, 1 MFMA
    int fuse;                    // 1: the O projection combines the attention partials itself (no combine tasks)
    int att_mc;                  // 1: attention tasks run on the matrix cores (kernels of the matrix-core path only)
    int ring_pages, page_bytes, n_stage;  // Eq. 1-2 outcome (0 pages: weights go straight to registers)
};

struct MatGeom {             // tile-major geometry of one matrix under a tiling
    int rlog, R, ck;         // rows per chunk, k per chunk (512 / R)
    int groups;              // row groups (of R rows)
    int kbt;                 // chunks per row group
    int n_rows, k_len;       // true output rows and K
    int w4;                  // 4-bit codes: ck = 2048 / R instead of 512 / R
    int S;                   // K slices per row group
    int sm;                  // 1: units and chunks are numbered K slice first (mk::unit_place)
};

struct Geom {
    MatGeom qkv, o, gu, down, head;
    int ipad;                // intermediate padded so that gate and up fill whole half groups
};

struct WeightMap {           // chunk / element offsets inside the workspace
    std::vector<uint32_t> qkv, o, gu, down;   // first chunk per layer
    uint32_t embed, head;
    std::vector<uint32_t> g_attn, g_mlp, bias, qn, kn;  // bf16 element offsets per layer (kNone if absent)
    uint32_t g_final;
    uint64_t n_chunks, n_vec;
    uint64_t n_layer_chunks;                  // chunks of the decoder layers (they come first; W4 scales cover exactly these)
};

struct ActMap {              // float offsets inside the activation region
    uint32_t xa, xb, pqkv, attp, o, po, gu, pd;   // gu holds silu(gate)*up when the gate/up epilogue is fused
    uint32_t amax;                                // arg-max partials [LM-head task slot][sequence][2] = (max logit, row)
    uint64_t n_floats;
};

struct SimResult {
    double makespan_us, duty;
};

}  // namespace mk

struct mk_schedule {
    mk_config cfg;
    mk::Dims dm;
    mk::Tiling tl;
    mk::Geom gm;
    mk::WeightMap wm;
    mk::ActMap am;
    mk::Layout lay;
    uint32_t lds_red_bytes, lds_xs_off, lds_total, lds_ring_off, lds_ring_slots;
    int n_wg, max_instr, n_counters, n_tasks;
    std::vector<uint32_t> instr;          // [n_wg][max_instr][32]
    std::vector<uint32_t> ref_seqs;       // distinct operator-instance ranks in topological order
    mk::SimResult sim;
    int cand_tried, cand_pruned;
    int from_table;          // 1: the tiling came from the table of recorded profile-guided tilings
    // ---- run-time binding (filled by mk_bind_workspace / mk_load_weights)
    char *ws;
    size_t ws_bytes;
    int device;
    bool bound, loaded;
    uint32_t epoch;
    void *ev0, *ev1;
    bool ev_valid;
    uint64_t serial;         // identity of this handle among the users of a GPU's static scratch array (0: not yet drawn)
    bool last_static;        // the most recent step ran on the static scratch array (mk_check reads the flags there)
};

namespace mk {
void set_error(const std::string &msg);
int build_schedule(const mk_config *cfg, mk_schedule **out);   // n_workgroups must be > 0 here
int verify_schedule(const mk_schedule *s);
int dump_schedule(const mk_schedule *s, void *buf, size_t *bytes);
int load_schedule(const void *buf, size_t bytes, mk_schedule **out);
int64_t pages_available(int64_t smem_max, int64_t n_stage, int64_t instr_buf, int64_t semaphores,
                        int64_t scratch, int64_t page_size);
int64_t pipeline_stages(int64_t pages_total, int64_t pages_weight, int64_t pages_scale, int64_t pages_act,
                        int64_t pages_per_stage);
}  // namespace mk
