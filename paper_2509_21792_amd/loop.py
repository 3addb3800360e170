"""Host driver of one speculative round and of the generation loop (Alg. 1, the generation loop).

Host bookkeeping only: it strings the library's entry points together (plan -> draft steps -> frontier updates ->
rerank -> verify -> accept -> compact), keeps every intermediate on the device, and crosses to the host once
per round for the accepted tokens, as the method requires to update the live set.
"""
import numpy as np
import torch

from . import binding as fg


class SpecState:
    """Per-batch device state carried between rounds: the entries the draft head has not seen yet."""

    def __init__(self, catch_tok, catch_feat, n_valid_minus1):
        self.catch_tok = catch_tok          # int32 [B, Kin]  token t+1 of each pending entry (padding beyond n_valid)
        self.catch_feat = catch_feat        # dtype [B, Kin, d] the target's feature t paired with it
        self.last = n_valid_minus1          # int32 [B] index of the last valid entry (= the root's entry)


def chain_parent(B, n, device):
    return torch.arange(-1, n - 1, dtype=torch.int32, device=device).repeat(B, 1)


def draft_expand(target, draft, dkv, slot, st, K, L, ws, max_seq_len=0):
    """L drafting steps, K paths kept per step.  Returns the candidate lists (tok, parent, score) [B, 1+K+(L-1)K^2]."""
    B, Kin = st.catch_tok.shape
    dev = st.catch_tok.device
    n_total = 1 + K + (L - 1) * K * K
    cand_tok = torch.empty((B, n_total), dtype=torch.int32, device=dev)
    cand_parent = torch.empty((B, n_total), dtype=torch.int32, device=dev)
    cand_score = torch.empty((B, n_total), dtype=torch.float32, device=dev)
    # step 1: the catch-up chain; its last valid row is the root, whose K best children open the tree
    ctok, clogp, ofeat = fg.fg_draft_step(target, draft, dkv, slot, st.catch_tok, chain_parent(B, Kin, dev), st.catch_feat, ws,
                                          K, n_commit=st.last, commit_bias=1, max_seq_len=max_seq_len, expand_row=st.last)
    f_tok, f_cand, f_score, f_src, parents = fg.fg_draft_frontier(ctok, clogp, 1, cand_tok, cand_parent, cand_score,
                                                                 node_pick=st.last, node_tok=st.catch_tok)
    n_cand = 1 + K
    feat_base = ofeat                      # [B, rows, d]: hidden states of the previous step's nodes
    for step in range(2, L + 1):
        n_prev = (step - 2) * K
        ctok, clogp, ofeat = fg.fg_draft_step(target, draft, dkv, slot, f_tok, parents, feat_base, ws, K, n_prev=n_prev,
                                              feat_index=f_src, max_seq_len=max_seq_len)
        f_tok, f_cand, f_score, f_src, parents = fg.fg_draft_frontier(ctok, clogp, n_cand, cand_tok, cand_parent, cand_score,
                                                                     node_cand=f_cand, node_score=f_score,
                                                                     parent_prev=parents)
        feat_base = ofeat
        n_cand += K * K
    return cand_tok, cand_parent, cand_score


def spec_round(target, draft, kv, dkv, slot, st, N, K, L, ws_t, ws_d, eos_id=-1, max_seq_len=0):
    """One round on the live batch.  Returns (accept_len, out_tokens, finished) on the device and the next SpecState."""
    ct, cp, cs = draft_expand(target, draft, dkv, slot, st, K, L, ws_d, max_seq_len=max_seq_len)
    tokens, parent, _ = fg.fg_build_tree(ct, cp, cs, ct.shape[1], N)
    out = fg.fg_spec_verify(target, kv, slot, tokens, parent, ws_t, max_seq_len=max_seq_len)
    acc, path, otok, fin = fg.fg_spec_accept(tokens, parent, row_argmax=out["argmax"], eos_id=eos_id)
    B = tokens.shape[0]
    d = target.cfg["d_model"]
    feat = fg.fg_kv_compact(kv, slot, acc, path, feature_in=out["feature"].view(B, N, d), d_model=d)
    Kin = L + 1
    nxt = SpecState(otok[:, :Kin].contiguous(), feat[:, :Kin].contiguous(), acc)
    return acc, otok, fin, nxt
