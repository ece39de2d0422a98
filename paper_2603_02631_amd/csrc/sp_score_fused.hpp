// Host interface of the fused single-launch score kernel (see sp_score_fused.hip).
#pragma once

#include "sp_common.hpp"
#include "sp_score_dev.hpp"

namespace sp_fused {

constexpr int kTileKeys = 512;   // keys owned by one workgroup at head_dim 64; 256 at head_dim 128
constexpr int kMaxRowsWide = 32; // head_dim 128: padded query rows per kv head
constexpr int kMaxRows = 64;     // padded query rows per kv head the kernel holds on chip
constexpr int kSlots = 8;        // depth of the exchange ring
constexpr int kMinWorkgroups = 64;       // head_dim 64: shorter prompts are faster on the two-pass path
constexpr int kMinWorkgroupsWide = 96;   // head_dim 128 (measured crossover near 24K tokens)
constexpr int kMaxGroupPrompts = 32;   // prompts one launch can serve

// Prompts of a ragged batch that share a launch: prompt i of the group is prompt `prompt[i]` of the
// batch (its queries), owns keys [start[i], start[i] + len[i]) of the packed key arrays (len >= one
// tile) and workgroups w0[i] .. w0[i+1]-1. n == 0: a single prompt described by FusedArgs::L.
struct GroupTable {
    int32_t n;
    int32_t w0[kMaxGroupPrompts + 1];
    int32_t prompt[kMaxGroupPrompts];
    int64_t start[kMaxGroupPrompts];
    int64_t len[kMaxGroupPrompts];
};

struct FusedArgs {
    const uint16_t *q;           // [Lyr][H][n_q][head_dim]
    int32_t head_dim;            // 64 or 128
    int32_t tile_keys;           // keys per workgroup: 512 at head_dim 64, 256 at head_dim 128
    int64_t k_stride_token, k_stride_head;
    int64_t L;
    uint64_t *part;              // [kSlots][n_wg][rows_pad]  (max, sum exp) partials, parity in bit 63
    uint64_t *lse;               // [kSlots][rows_pad]        (-lse, phase + 1)
    uint32_t *err;               // the call's status word: raised by any workgroup whose bounded wait gave up
    uint32_t spin_max;           // polls before a wait gives up
    int32_t force_miss;          // test hook: duty waves treat their partials as never arriving
    const float *kscale;         // 8-bit keys (E4M3 codes): [n_phases] scale of each (layer, kv head); null: bf16 keys
    const float *look;           // [n_phases][rows_pad] log-sum-exp of each row over its visible lookahead keys
                                 // (raw-logit units, -inf for none), or null: prompt keys only
    const int32_t *block_table;  // paged keys: token j of a layer sits in page block_table[j / page_tokens] of that
    int64_t page_tokens;         // layer's pool, page p at element offset p * page_stride; null: contiguous keys
    int64_t page_stride;
    float *scores;
    int32_t n_wg;
    int32_t n_gp, p_idx;         // set in the kernel: prompts in the launch, this workgroup's prompt among them
    int32_t n_layers, n_q_heads, n_kv_heads, group, n_q;
    int32_t n_nblk, n_gblk, rows_pad;
    int32_t layer_agg;
    float c, inv_c, out_scale;
};

size_t workspace_bytes(int rows_pad, int n_wg, int n_prompts);

// True when the device can hold one workgroup of the fused kernel per compute unit.
bool fits_one_per_cu();

// Enqueues the clear kernel and the fused kernel. `ws` must hold workspace_bytes(); `status_word`
// (device) is cleared first and raised if the call gives up.
// `group` (or null for one prompt) describes the prompts of the launch; the status word is cleared only
// when clear_status is set (the first launch of a call).
sp_status launch(FusedArgs a, const sp_dev::LayerPtrs &kp, const GroupTable *group, bool clear_status, void *ws,
                 uint32_t *status_word, hipStream_t st);

// Test hook: polls before a bounded wait gives up (default 2^20) and whether duty waves treat their
// partials as never arriving; applies to launches that follow.
void set_giveup(uint32_t spin_max, int32_t force_miss);

}  // namespace sp_fused
