"""Graph templates written against the registrar primitives (add_dim / add_chunk_param / add_tensor / add_op /
add_alias / add_barrier).  A template function takes any builder exposing those methods, so the same
description instantiates the library's registrar and the test oracle's; it holds no planning arithmetic.

Paper section 4.3 describes templates of this kind (topology and memory dependencies written down once, the
input-dependent dimensions left symbolic); the operator list below is a reduced dLLM denoising step with the
two operators the paper chunks (section 4.4): the feed-forward network over all T tokens and the logits over
the M masked tokens.
"""

NONE = -1


def dllm_step(b, layers=2, d=64, d_ff=256, vocab=1024, logits="materialised", vocab_splits=16, inplace_residual=True):
    """Reduced denoising step.  bf16 activations (2 bytes), fp32 logits (4 bytes).

    logits = "materialised": the logits operator writes an [M/K, V] fp32 tensor that the sampling operator
    reads (the paper's design).  logits = "fused": it writes 12 bytes of partial results per row and
    vocabulary split (this library's fused kernel), so its workspace is independent of V.
    Returns a dict of the ids a caller may want (dims, chunk parameters, a few tensors)."""
    T = b.add_dim("T")
    M = b.add_dim("M")
    k_ffn = b.add_chunk_param("K_ffn", T)
    k_logits = b.add_chunk_param("K_logits", M)
    tokens = b.add_tensor("tokens", 4, T, NONE, True)
    h = b.add_tensor("h0", 2 * d, T, NONE, False)
    b.add_op("embed", [tokens], [h], NONE)
    for l in range(layers):
        qkv = b.add_tensor(f"qkv{l}", 3 * 2 * d, T, NONE, False)
        att = b.add_tensor(f"att{l}", 2 * d, T, NONE, False)
        mid = b.add_tensor(f"mid{l}", 2 * d, T, NONE, False)
        gate_up = b.add_tensor(f"gate_up{l}", 2 * 2 * d_ff, T, k_ffn, False)
        act = b.add_tensor(f"act{l}", 2 * d_ff, T, k_ffn, False)
        nxt = b.add_tensor(f"h{l + 1}", 2 * d, T, NONE, False)
        b.add_op(f"qkv_proj{l}", [h], [qkv], NONE)
        b.add_op(f"attention{l}", [qkv], [att], NONE)
        b.add_op(f"out_proj{l}", [att, h], [mid], NONE)
        if inplace_residual:
            b.add_alias(h, mid)                  # the residual sum is written over its input
        b.add_op(f"ffn_up{l}", [mid], [gate_up], k_ffn)
        b.add_op(f"ffn_act{l}", [gate_up], [act], k_ffn)
        b.add_op(f"ffn_down{l}", [act, mid], [nxt], k_ffn)
        h = nxt
    hn = b.add_tensor("h_norm", 2 * d, T, NONE, False)
    b.add_op("final_norm", [h], [hn], NONE)
    idx = b.add_tensor("mask_idx", 4, M, NONE, False)
    b.add_op("mask_compact", [tokens], [idx], NONE)
    out = b.add_tensor("token_conf_lse", 12, M, NONE, False)
    if logits == "materialised":
        lg = b.add_tensor("logits", 4 * vocab, M, k_logits, False)
        b.add_op("lm_head", [hn, idx], [lg], k_logits)
        b.add_op("sample", [lg], [out], k_logits)
    elif logits == "fused":
        part = b.add_tensor("partials", 12 * vocab_splits, M, k_logits, False)
        b.add_op("lm_head_reduce", [hn, idx], [part], k_logits)
        b.add_op("merge_splits", [part], [out], k_logits)
    else:
        raise ValueError(logits)
    b.add_op("unmask", [out, idx, tokens], [tokens], NONE)
    return dict(T=T, M=M, k_ffn=k_ffn, k_logits=k_logits, h_norm=hn, out=out)


def mask_only_tail(b, vocab_splits, scan_scratch_bytes, partial_bytes=12, row_tile=256, sync_bytes=1024):
    """The tail of a denoising step that this library runs, as a template: mask compaction, the fused LM-head
    reduction in K_logits chunks over masked rows, the split merge, top-n unmasking.  Hidden states, LM head, mask
    and token sequence are the step's inputs (persistent: outside the workspace).

    The masked-row dimension is counted in ROW TILES (R = ceil(M / row_tile)), because the kernel's chunk size is a
    whole number of row tiles: a chunk of ceil(R / K) tiles holds partial_bytes * vocab_splits * row_tile bytes of
    partial results per tile; the fixed sync_bytes of round counters that close the fused call's workspace are
    counted once per tile, so that a chunk's block is never smaller than what the call asks for.  partial_bytes is
    12 for the greedy reduction, 20 for temperature sampling.  Returns the ids a caller needs to find the buffers in a plan."""
    T = b.add_dim("T")
    R = b.add_dim("R")
    k_logits = b.add_chunk_param("K_logits", R)
    mask = b.add_tensor("mask", 1, T, NONE, True)
    hidden = b.add_tensor("hidden", 2, T, NONE, True)
    tokens = b.add_tensor("tokens", 4, T, NONE, True)
    idx = b.add_tensor("mask_idx", 4, T, NONE, False)
    count = b.add_tensor("mask_count", 4, NONE, NONE, False)
    scratch = b.add_tensor("scan_scratch", max(int(scan_scratch_bytes), 1), NONE, NONE, False)
    partials = b.add_tensor("partials", partial_bytes * vocab_splits * row_tile + sync_bytes, R, k_logits, False)
    out_token = b.add_tensor("out_token", 4 * row_tile, R, NONE, False)
    out_conf = b.add_tensor("out_conf", 4 * row_tile, R, NONE, False)
    out_lse = b.add_tensor("out_lse", 4 * row_tile, R, NONE, False)
    b.add_op("mask_compact", [mask], [idx, count, scratch], NONE)
    b.add_op("lm_head_reduce", [hidden, idx, count], [partials], k_logits)
    b.add_op("merge_splits", [partials, count], [out_token, out_conf, out_lse], k_logits)
    b.add_op("unmask", [out_token, out_conf, idx, count, mask, tokens], [tokens, mask], NONE)
    return dict(T=T, R=R, k_logits=k_logits, idx=idx, count=count, scratch=scratch, partials=partials,
                out_token=out_token, out_conf=out_conf, out_lse=out_lse)
