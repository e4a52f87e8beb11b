// Internal launch interface between the C-ABI layer (api.hip) and the kernel files.
#pragma once

#include "common.h"

namespace omni {

// score.hip
size_t score_queries_ws(const Layer& L);
int run_score_queries(const Layer& L, int dtype, const void* Q, const void* K, float* probe, float* scores, void* ws,
                      hipStream_t st);
int run_probe_keys(const Layer& L, int dtype, const void* K, float* probe, void* ws, hipStream_t st);

// select.hip
size_t select_ws(const Layer& L);
int run_select_queries(const Layer& L, const float* scores, int mode, float param, int* q_idx, int* q_cnt, void* ws,
                       hipStream_t st);
int run_select_kv(const Layer& L, const float* key_scores, const int* budget, int b_cap, int* kv_idx, void* ws,
                  hipStream_t st);
size_t budget_stats_ws(const Layer& L);
int run_budget_stats(const Layer& L, const float* key_scores, float recall_p, int budget_mode, double* kurt,
                     int* flattest, int* budget, float* recall, void* ws, hipStream_t st, int k_cap = 0x7fffffff);
int run_select_kv_from_stats(const Layer& L, const float* key_scores, void* stats_ws, int b_cap, int* kv_idx,
                             void* ws, hipStream_t st);
// The key lists as the packing kernel can form them itself: the scores, each head's cut (threshold key and number of
// cut-valued elements to take) and, per chunk of kSelectChunk elements, how many kept elements precede it.  out
// receives the lists ([B*Hq, out_stride], what run_select_kv_from_stats writes).
constexpr int kSelectChunk = 1024;
struct SelectSource {
  const float* x;          // [B*Hq, ld]
  int ld, nchunk;
  const unsigned* thr;     // [B*Hq]
  const int* need;         // [B*Hq]
  const int* off_keep;     // [B*Hq, nchunk] exclusive counts of elements above the cut
  const int* off_eq;       // [B*Hq, nchunk] exclusive counts of elements at the cut
  int* out;
  int out_stride;
};
// the counting half of run_select_kv_from_stats: fills *src (pointers into the two workspaces), writes no list
int run_select_kv_counts(const Layer& L, const float* key_scores, void* stats_ws, int b_cap, int* kv_idx, void* ws,
                         SelectSource* src, hipStream_t st);
int run_visual_subset(const Layer& L, const int* kv_idx, const int* budget, int b_cap, int* vis_idx, int* vis_cnt,
                      hipStream_t st);
size_t group_subset_ws(const Layer& L);
int run_group_subset(const Layer& L, const int* kv_idx, const int* budget, int b_cap, int* grp_idx, unsigned* grp_mask,
                     int* grp_cnt, int u_cap, void* ws, hipStream_t st);

// probe.hip
size_t probe_ws(const Layer& L, int dtype, int pb);
// probe_keys / scores not null: the pooling pass over Q also writes the lazy/active query scores
int run_probe(const Layer& L, int dtype, const void* Q, const void* K, int pb, float* key_scores, void* ws,
              hipStream_t st, const float* probe_keys = nullptr, float* scores = nullptr);

// pack.hip (outputs that are nullptr are skipped; Kt / Vt / Qt / dOt exist for bf16 only; Vt holds f16 values)
// sel not null (per_q_head only, src_idx ignored): the kernel forms the lists from *sel and writes them to sel->out
int run_pack_kv(const Layer& L, int dtype, const void* K, const void* V, int per_q_head, const int* src_idx,
                int idx_stride, const int* budget, int b_cap, int npad, int pad_to, void* Kn, void* Vn, void* Kt,
                void* Vt, int* kidx, hipStream_t st, const SelectSource* sel = nullptr);
int run_pack_q(const Layer& L, int dtype, const void* Q, const void* O, const void* dO, const float* lse,
               const int* q_idx, const int* q_cnt, int nqpad, void* Qt, void* dOt, void* Qn, void* dOn, float* lse2c,
               float* deltac, hipStream_t st);

// qvis [B*Hq, N] / kfirst [B*Hq, npad] (either may be nullptr): visibility bounds of the causal mask on the
// packed, ascending key and kept-query lists of every query head
int run_visible_counts(const Layer& L, const int* q_idx, const int* q_cnt, const int* kidx, const int* budget,
                       int b_cap, int npad, int* qvis, int* kfirst, hipStream_t st);

// attn_fwd.hip
size_t attn_fwd_ws(const Layer& L, int dtype, int b_cap, bool sparse);
// sel not null: kv_idx is an output, formed from *sel by the packing kernel (sparse only)
int run_attn_fwd(const Layer& L, int dtype, const void* Q, const void* K, const void* V, const int* q_idx,
                 const int* q_cnt, const int* kv_idx, const int* budget, int b_cap, void* O, float* lse, void* ws,
                 bool sparse, hipStream_t st, const SelectSource* sel = nullptr);

// bf16 only, block % 64 == 0: the forward pass on block lists without a gathered copy of K/V per query head
int attn_fwd_blocks_max_keys();
// tile_map[bh, t] = tile of the KV head's token-ordered K/V copy that holds tile t of the head's block list
int run_tile_map(const Layer& L, const int* blk_idx, const int* blk_budget, int blk_cap, int block, int last_tile,
                 int* tile_map, hipStream_t st);
size_t attn_fwd_blocks_ws(const Layer& L, int cap_keys);   // cap_keys = blk_cap * block
int run_attn_fwd_blocks(const Layer& L, const void* Q, const void* K, const void* V, const int* q_idx, const int* q_cnt,
                        const int* blk_idx, const int* blk_budget, int blk_cap, int block, void* O, float* lse,
                        void* ws, hipStream_t st);

// attn_bwd.hip
size_t attn_bwd_ws(const Layer& L, int dtype, int b_cap);
int run_attn_bwd(const Layer& L, int dtype, const void* Q, const void* K, const void* V, const void* O,
                 const void* dO, const float* lse, const int* q_idx, const int* q_cnt, const int* kv_idx,
                 const int* budget, int b_cap, void* dQ, void* dK, void* dV, void* ws, hipStream_t st);
// the same on block lists walked in place (bf16): K/V of every KV head once, tiles found through a tile map
int attn_bwd_blocks_max_keys();
size_t attn_bwd_blocks_ws(const Layer& L, int cap_keys);   // cap_keys = blk_cap * block
int run_attn_bwd_blocks(const Layer& L, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                        const float* lse, const int* q_idx, const int* q_cnt, const int* blk_idx, const int* blk_budget,
                        int blk_cap, int block, void* dQ, void* dK, void* dV, void* ws, hipStream_t st);

void set_key_split_len(int tiles);   // attn_bwd.hip; <= 0 restores the default

// decode.hip
size_t decode_ws(const omni_decode_desc* d);
// paged form of the compacted store: Kcomp / Vcomp are a pool [pool_pages, 1 << page_shift, D] shared by all
// (batch, KV head) pairs; position u of a pair's group list lives in page page_table[pair, u >> page_shift]
struct PagePool {
  const int* page_table;   // [B*Hkv, pages_cap]; entries outside [0, pool_pages) mark pages that are not there
  int page_shift, pages_cap, pool_pages;
};
// grp_mask == nullptr: vis_idx / vis_cnt are per query head; otherwise per KV group with membership bits
int run_decode(const omni_decode_desc* d, const void* q, const void* K, const void* V, const int* ctx_len,
               const float* probe, const int* vis_idx, const int* vis_cnt, const unsigned* grp_mask, int b_cap,
               void* O, unsigned char* active, void* ws, hipStream_t st, const void* Kcomp = nullptr,
               const void* Vcomp = nullptr, const PagePool* pool = nullptr);
int run_compact_cache(const omni_decode_desc* d, const void* K, const void* V, const int* grp_idx, const int* grp_cnt,
                      int u_cap, void* Kc, void* Vc, hipStream_t st, const PagePool* pool = nullptr);

// block.hip (block-granular variant of the KV selection)
int block_scores_max_blocks();
size_t block_scores_ws(const Layer& L, int block);
int run_block_scores(const Layer& L, int dtype, const void* Q, const void* K, int block, float* out, void* ws,
                     hipStream_t st);
int run_expand_blocks(const Layer& L, const int* blk_idx, const int* blk_budget, int blk_cap, int block, int* kv_idx,
                      int* budget, int b_cap, hipStream_t st);

// diag.hip
int run_calibration_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
int run_mfma_rate(int random_operands, int iters, double* tflops, double* shader_mhz);

}  // namespace omni
