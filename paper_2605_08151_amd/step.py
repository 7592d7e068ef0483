"""One verification step = the four library calls in order, with their scratch buffers.

Glue for tests and the benchmark: owns torch-allocated workspaces and outputs, nothing numerical.
"""
from __future__ import annotations

import torch

from . import binding as sv


class VerifyStep:
    def __init__(self, B, M, Hq, Hkv, D, H, V, gamma_max, max_kv_len, device="cuda"):
        self.B, self.M, self.Hq, self.Hkv, self.D, self.H, self.V = B, M, Hq, Hkv, D, H, V
        self.gamma_max, self.max_kv_len = gamma_max, max_kv_len
        dev = torch.device(device)
        self.attn_ws = torch.empty(max(256, sv.spec_verify_attn_workspace_bytes(B, M, Hq, Hkv, D, max_kv_len, gamma_max + 1)),
                                   dtype=torch.uint8, device=dev)
        self.accept_ws = torch.empty(max(256, sv.spec_accept_workspace_bytes(B, M, V, gamma_max)), dtype=torch.uint8, device=dev)
        self.attn_out = torch.empty((M, Hq, D), dtype=torch.bfloat16, device=dev)
        self.lse = torch.empty((M, Hq), dtype=torch.float32, device=dev)
        self.logits = torch.empty((M, V), dtype=torch.float32, device=dev)
        self.accept_len = torch.empty(B, dtype=torch.int32, device=dev)
        self.out_tokens = torch.empty((B, gamma_max + 1), dtype=torch.int32, device=dev)
        self.rollback = torch.empty(B, dtype=torch.uint8, device=dev)
        self.stats = torch.zeros(4, dtype=torch.int32, device=dev)
        self.status = torch.zeros(1, dtype=torch.int32, device=dev)
        # block statistics of the fused LM head (0 blocks: the shape has none and acceptance scans the logits)
        self.blocks = sv.spec_lm_head_stats_blocks(M, H, V)
        self.blk_max = torch.empty((M, max(1, self.blocks)), dtype=torch.float32, device=dev)
        self.blk_arg = torch.empty((M, max(1, self.blocks)), dtype=torch.int32, device=dev)
        # the same for the packed LM head (its blocks are the passes of its workgroups)
        self.pblocks = sv.spec_lm_head_packed_stats_blocks(M, H, V)
        self.pblk_max = torch.empty((M, max(1, self.pblocks)), dtype=torch.float32, device=dev)
        self.pblk_arg = torch.empty((M, max(1, self.pblocks)), dtype=torch.int32, device=dev)

        # block summaries of the large-tile packed LM head (more than 160 rows): maxima and sums per block of 64 entries
        self.sblocks = sv.spec_lm_head_packed_summary_blocks(M, H, V)
        self.sblk_max = torch.empty((M, max(1, self.sblocks)), dtype=torch.float32, device=dev)
        self.sblk_sum = torch.empty((M, max(1, self.sblocks)), dtype=torch.float32, device=dev)
        self.sblk_span = torch.empty((max(1, self.sblocks), 2), dtype=torch.int32, device=dev)

    def lm_head_packed_summary(self, hidden, Wp, temperature, qo_indptr):
        sv.spec_lm_head_packed_summary(hidden, Wp, self.logits, temperature, qo_indptr, self.sblk_max, self.sblk_sum, self.sblk_span)
        return self.logits

    def accept_summary(self, tokens, draft_probs, temperature, seeds, round_, qo_indptr):
        sv.spec_accept_summary(self.logits, tokens, draft_probs, temperature, seeds, round_, qo_indptr, self.accept_len,
                               self.out_tokens, self.rollback, self.stats, self.gamma_max, self.sblk_max, self.sblk_sum,
                               self.sblk_span, self.sblocks, self.status, self.accept_ws)
        return self.accept_len, self.out_tokens

    def attn(self, q, k_cache, v_cache, page_table, seq_lens, qo_indptr, scale, want_lse=True):
        sv.spec_verify_attn(q, k_cache, v_cache, page_table, seq_lens, qo_indptr, self.attn_out,
                            self.lse if want_lse else None, self.max_kv_len, self.gamma_max + 1, scale, self.status,
                            self.attn_ws)
        return self.attn_out

    def lm_head(self, hidden, W):
        sv.spec_lm_head(hidden, W, self.logits)
        return self.logits

    def pack_weights(self, W):
        """The vocabulary matrix in the layout spec_lm_head_packed reads (done once, when the model is loaded)."""
        Wp = torch.empty(sv.spec_lm_head_packed_bytes(self.V, self.H) // 2, dtype=torch.bfloat16, device=W.device)
        sv.spec_lm_head_pack(W, Wp)
        return Wp

    def lm_head_packed(self, hidden, Wp):
        sv.spec_lm_head_packed(hidden, Wp, self.logits)
        return self.logits

    def lm_head_packed_stats(self, hidden, Wp):
        sv.spec_lm_head_packed_stats(hidden, Wp, self.logits, self.pblk_max, self.pblk_arg)
        return self.logits

    def accept_packed_stats(self, tokens, draft_probs, temperature, seeds, round_, qo_indptr):
        sv.spec_accept_stats(self.logits, tokens, draft_probs, temperature, seeds, round_, qo_indptr, self.accept_len,
                             self.out_tokens, self.rollback, self.stats, self.gamma_max, self.pblk_max, self.pblk_arg,
                             self.pblocks, self.status, self.accept_ws)
        return self.accept_len, self.out_tokens

    def lm_head_stats(self, hidden, W):
        sv.spec_lm_head_stats(hidden, W, self.logits, self.blk_max, self.blk_arg)
        return self.logits

    def accept_stats(self, tokens, draft_probs, temperature, seeds, round_, qo_indptr):
        sv.spec_accept_stats(self.logits, tokens, draft_probs, temperature, seeds, round_, qo_indptr, self.accept_len,
                             self.out_tokens, self.rollback, self.stats, self.gamma_max, self.blk_max, self.blk_arg,
                             self.blocks, self.status, self.accept_ws)
        return self.accept_len, self.out_tokens

    def accept(self, tokens, draft_probs, temperature, seeds, round_, qo_indptr, logits=None):
        sv.spec_accept(self.logits if logits is None else logits, tokens, draft_probs, temperature, seeds, round_,
                       qo_indptr, self.accept_len, self.out_tokens, self.rollback, self.stats, self.gamma_max,
                       self.status, self.accept_ws)
        return self.accept_len, self.out_tokens

    def commit(self, page_table, seq_lens, qo_indptr, free_list, free_count, page_size=16):
        sv.spec_kv_commit(page_table, seq_lens, qo_indptr, self.accept_len, free_list, free_count, page_size, self.status)
