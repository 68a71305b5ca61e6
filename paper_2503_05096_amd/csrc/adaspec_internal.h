// Internal declarations shared by the translation units of libadaspec.so:
// workspace layouts and the launchers each kernel file exports.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/adaspec.h"

namespace adaspec {

// ---- attention workspace -------------------------------------------------
// A "work item" is one (request, KV split); splits of a request have equal
// length (a multiple of the kernel's token block).  Items are stored densely
// in request order; the plan kernel builds the list on the device because the
// context lengths live there.
struct AttnPlan {
    int   split_tokens;     // S: maximum tokens per split
    int   block_tokens;     // split lengths are rounded up to a multiple of this
    int   max_items;        // host-side bound on the number of work items
    int   max_rows;         // (max_spec_len + 1) * G
    // byte offsets into the workspace
    size_t off_header;      // int32[16]: [0] n_items, [1] unused, [2] rounds of the static schedule
    size_t off_cu_q;        // int32[B + 1]
    size_t off_split_base;  // int32[B + 1]: first item of each request
    size_t off_item_req;    // int32[max_items]
    size_t off_item_order;  // int32[max_items]: items sorted by decreasing length (schedule order)
    size_t off_unit_meta;   // int32[max_items][8] in schedule order: request, split, n_splits, L, n, cu_q, item, 0
    size_t off_row_rec;     // int32[TQ][4] per query row: request, n_splits, first split, row base (j * G)
    size_t off_sched;       // int32[rounds][W]: unit taken by workgroup w in each round, or -1 (matrix-core kernel)
    size_t off_anc;         // uint64[TQ]: tree verification only, ancestor-or-self mask of each query row's node
    size_t off_part_ml;     // float[max_items][Hkv][max_rows][2]  (m in log2 units, l)
    size_t off_part_o;      // float[max_items][Hkv][max_rows][d]
    size_t total_bytes;
};

// Length of every split of a request with L cached tokens cut into ns splits.
__host__ __device__ inline int split_len_of(int L, int ns, int block_tokens)
{
    const int per = (L + ns - 1) / ns;
    return (per + block_tokens - 1) / block_tokens * block_tokens;
}

// Matrix-core kernels: 16-row query tiles one unit holds and units per (item, kv head).  Up to 32 rows per
// kv head: 1 or 2 tiles, the wavefronts of a workgroup split the unit's tokens (attn_mfma.hip); more: groups
// of 4 tiles (64 rows), the wavefronts split the rows (attn_rows.hip).
inline int attn_row_tiles(int max_rows)
{
    return max_rows <= 16 ? 1 : (max_rows <= 32 ? 2 : 4);
}
inline int attn_row_groups(int max_rows)
{
    const int r = 16 * attn_row_tiles(max_rows);
    return max_rows > r ? (max_rows + r - 1) / r : 1;
}

AttnPlan make_attn_plan(const adaspec_attn_dims &d, bool fast_path);
bool attn_fast_path_supported(const adaspec_attn_dims &d);

struct AttnArgs {
    const void *q, *k_pages, *v_pages;
    const int32_t *block_table, *ctx_lens, *spec_lens;
    const int32_t *parents = nullptr;   // tree verification: parent node of every query row, else NULL
    void *out;
    adaspec_attn_dims dims;
    float scale_log2;       // scale * log2(e)
    AttnPlan plan;
    char *ws;
    hipStream_t stream;
    // launch shape of the matrix-core kernel (attn_mfma_shape); sched_w = 0 on the vector path
    int sched_w = 0;          // W: workgroups of the launch = columns of the schedule table
    int sched_cus = 1;        // compute units of the device
    int n_row_groups = 1;     // units per (item, kv head)
    int rows_per_group = 16;  // query rows (times G) one unit covers
};

// Upper bound on W for which the workspace holds a schedule table.
constexpr int kMaxSchedW = 1024;
constexpr int64_t kMaxAttnItems = (int64_t)1 << 24;   // (request, split) work items of one attention call

// Fills sched_w / n_row_groups / rows_per_group for the matrix-core kernel's launch of a.dims.
void attn_mfma_shape(AttnArgs &a);

hipError_t launch_attn_plan(const AttnArgs &a);
// tree verification: ancestor masks of all query rows (after the plan kernel: it reads cu_q)
hipError_t launch_tree_masks(const AttnArgs &a);
hipError_t launch_attn_vector(const AttnArgs &a);
hipError_t launch_attn_mfma(const AttnArgs &a);
// row-split form for units of more than 32 rows (attn_rows.hip); launch_attn_mfma forwards to it
hipError_t launch_attn_rows(const AttnArgs &a);
int attn_rows_grid_slots(const AttnArgs &a, int cus);   // resident workgroups = columns of the schedule table
hipError_t launch_attn_combine(const AttnArgs &a);

// ---- accept workspace ------------------------------------------------------
struct AcceptPlan {
    size_t off_cu_q;        // int32[B + 1]
    size_t off_row_req;     // int32[TQ]
    size_t off_row_flag;    // int32[TQ]  1 = accepted (or bonus row)
    size_t off_row_cand;    // int32[TQ]  token to emit if the request stops at this row
    size_t off_row_meta;    // int32[TQ][8]: request, position j, k, draft token, temperature bits, draft row
    // two-pass form
    size_t off_row_stat;    // RowStat[TQ]: (m, Z) of the sampled draft rows, from the first pass (one workgroup per row)
    size_t off_req_ticket;  // int32[B]: workgroups of the second pass that have finished, per request
    size_t off_slot_rec;    // int32[B * max_spec_len][4] per (request, draft position): token, its logit, its draft
                            // probability, the accept uniform (form in parts)
    size_t off_part_stat;   // HalfStat[B * max_spec_len][8]: (maximum, normaliser | arg-max) of each part of a draft row
    size_t off_half_stat;   // HalfStat[B][16]: per part of the deciding row
    size_t off_part;        // float[B][16 parts][4 steps][4][2][4]: partial sums of the deciding rows
    size_t off_tree_stat;   // tree acceptance: per-node statistics (tree_node_stat_bytes() each)
    size_t total_bytes;
};
// p_v = 2^((l_v - m) c) / Z of a row (first pass of the two-pass form -> second pass)
struct RowStat { float m; float pad; double Z; };
// per part of a row: (m, Z) the part's sums are relative to; for a greedy row (maximum, arg-max or -1)
struct HalfStat { float m; int arg; double Z; };
AcceptPlan make_accept_plan(const adaspec_accept_dims &d);
bool accept_fast_path_supported(const adaspec_accept_dims &d, const void *logits, const void *probs);

struct AcceptArgs {
    const void *logits, *probs;
    const int32_t *draft_tokens;
    const float *uniforms;
    const int32_t *spec_lens;
    const float *temperature;
    int32_t *out_tokens, *out_accept_len;
    adaspec_accept_dims dims;
    AcceptPlan plan;
    char *ws;
    hipStream_t stream;
};

hipError_t launch_accept_plan(const AcceptArgs &a);
hipError_t launch_accept_vector(const AcceptArgs &a);
hipError_t launch_accept_fast(const AcceptArgs &a);
hipError_t launch_accept_emit(const AcceptArgs &a);
bool accept_stream_path_supported(const adaspec_accept_dims &d, const void *logits, const void *probs);
hipError_t launch_accept_stream(const AcceptArgs &a);
// two-pass form: flags of the draft rows, then one workgroup per request (sampling + outputs)
hipError_t launch_accept_test(const AcceptArgs &a);
hipError_t launch_accept_resolve(const AcceptArgs &a);
// two-pass form with every row cut into parts (accept_parts.hip): up to 1024 requests
bool accept_parts_supported(const adaspec_accept_dims &d);
size_t accept_parts_slot_bytes(const adaspec_accept_dims &d);
size_t accept_parts_stat_bytes(const adaspec_accept_dims &d);
size_t accept_parts_sum_bytes(const adaspec_accept_dims &d);
size_t accept_parts_sum_stat_bytes(const adaspec_accept_dims &d);
hipError_t launch_accept_parts(const AcceptArgs &a);

// tree verification (tree.hip, tree_fast.hip): every node's acceptance, then the walk; needs the accept plan's cu_q / row_req
// portable form (any types and sizes): a per-node kernel writes (next node or -1, token if the walk stops here)
// into row_flag / row_cand, a small kernel walks them
hipError_t launch_accept_tree_nodes(const AcceptArgs &a, const int32_t *parents);
// 16-bit rows (shapes of the register-resident chain kernel): node statistics, then one workgroup per request
// walks its tree and writes the outputs (no separate walk kernel)
size_t tree_node_stat_bytes();
bool tree_fast_needs_plan(const adaspec_accept_dims &d);   // large batches: row offsets from launch_accept_plan
hipError_t launch_accept_tree_fast(const AcceptArgs &a, const int32_t *parents, int32_t *out_path);
hipError_t launch_accept_tree_walk(const AcceptArgs &a, int32_t *out_path);
hipError_t launch_kv_compact_path(void *k_pages, void *v_pages, const int32_t *block_table,
                                  const int32_t *ctx_lens, const int32_t *spec_lens,
                                  const int32_t *out_path, const int32_t *out_accept_len,
                                  const adaspec_attn_dims &d, int path_stride, hipStream_t stream);

hipError_t launch_check_accept_inputs(const int32_t *draft_tokens, const int32_t *spec_lens, const float *temperature,
                                      const adaspec_accept_dims &d, int32_t *err_flags, hipStream_t stream);
hipError_t launch_check_tree_parents(const int32_t *parents, const int32_t *spec_lens, int B, int total_q,
                                     int max_spec_len, int32_t *err_flags, hipStream_t stream);
hipError_t launch_check_ragged(const int32_t *block_table, const int32_t *ctx_lens,
                               const int32_t *spec_lens, const adaspec_attn_dims &d,
                               int32_t *err_flags, hipStream_t stream);

bool draft_sample_supported(const adaspec_draft_dims &d, const void *logits, const void *probs);
hipError_t launch_draft_sample(const void *logits, const float *temperature, const float *uniforms,
                               const int32_t *out_rows, void *probs, int32_t *tokens, float *confidence,
                               const adaspec_draft_dims &d, hipStream_t stream);
bool draft_fast_supported(const adaspec_draft_dims &d);
// every row cut into four parts, three kernels (draft_split.hip); ws = draft_split_workspace_bytes(rows)
bool draft_split_supported(const adaspec_draft_dims &d);
size_t draft_split_workspace_bytes(int rows);
hipError_t launch_draft_split(const void *logits, const float *temperature, const float *uniforms,
                              const int32_t *out_rows, void *probs, int32_t *tokens, float *confidence,
                              const adaspec_draft_dims &d, char *ws, hipStream_t stream);
hipError_t launch_draft_fast(const void *logits, const float *temperature, const float *uniforms,
                             const int32_t *out_rows, void *probs, int32_t *tokens, float *confidence,
                             const adaspec_draft_dims &d, hipStream_t stream);
hipError_t launch_kv_append(const void *k_new, const void *v_new, void *k_pages, void *v_pages,
                            const int32_t *block_table, const int32_t *ctx_lens,
                            const int32_t *spec_lens, const adaspec_attn_dims &d, hipStream_t stream);
hipError_t launch_commit(const int32_t *out_tokens, const int32_t *out_accept_len,
                         const int32_t *spec_lens, const int32_t *ctx_lens,
                         const int32_t *next_spec_lens, int32_t *committed_lens,
                         int32_t *next_ctx_lens, int32_t *last_token, int32_t *seq_tokens,
                         int32_t *seq_lens, const adaspec_commit_dims &d, hipStream_t stream);

}  // namespace adaspec
