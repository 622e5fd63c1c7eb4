"""Tensor-size tables of the synthetic model states, in declaration order.

Only integers: (name, number of elements) per tensor.  These stand in for the
HuggingFace GPT-2 / LLaMA model states the paper trains (its Table 1 and
Experiment Setup); an optimizer step depends only on the sizes.
"""
from __future__ import annotations


def gpt2_block(h: int = 768, mlp: int | None = None, prefix: str = "h0."):
    mlp = 4 * h if mlp is None else mlp
    return [
        (prefix + "ln_1.weight", h), (prefix + "ln_1.bias", h),
        (prefix + "attn.c_attn.weight", h * 3 * h), (prefix + "attn.c_attn.bias", 3 * h),
        (prefix + "attn.c_proj.weight", h * h), (prefix + "attn.c_proj.bias", h),
        (prefix + "ln_2.weight", h), (prefix + "ln_2.bias", h),
        (prefix + "mlp.c_fc.weight", h * mlp), (prefix + "mlp.c_fc.bias", mlp),
        (prefix + "mlp.c_proj.weight", mlp * h), (prefix + "mlp.c_proj.bias", h),
    ]


def gpt2(h: int, n_blocks: int, mlp: int, vocab: int = 50257, n_pos: int = 1024):
    """Token + position embedding, blocks, final LayerNorm; the head is tied to the embedding."""
    out = [("wte.weight", vocab * h), ("wpe.weight", n_pos * h)]
    for i in range(n_blocks):
        out += gpt2_block(h, mlp, prefix=f"h{i}.")
    out += [("ln_f.weight", h), ("ln_f.bias", h)]
    return out


def llama(h: int, ffn: int, n_blocks: int, vocab: int = 32000):
    """Untied embedding and head, SwiGLU FFN, RMSNorm gains."""
    out = [("embed_tokens.weight", vocab * h)]
    for i in range(n_blocks):
        p = f"layers.{i}."
        out += [
            (p + "q_proj.weight", h * h), (p + "k_proj.weight", h * h),
            (p + "v_proj.weight", h * h), (p + "o_proj.weight", h * h),
            (p + "gate_proj.weight", h * ffn), (p + "up_proj.weight", h * ffn),
            (p + "down_proj.weight", ffn * h),
            (p + "input_layernorm.weight", h), (p + "post_attention_layernorm.weight", h),
        ]
    out += [("norm.weight", h), ("lm_head.weight", vocab * h)]
    return out


def block_ids(table):
    """Transformer-block id per tensor (None for tensors outside the blocks), from the names
    'h<i>.' (GPT-2) / 'layers.<i>.' (LLaMA)."""
    out = []
    for name, _ in table:
        head = name.split(".")
        if head[0].startswith("h") and head[0][1:].isdigit():
            out.append(int(head[0][1:]))
        elif head[0] == "layers" and len(head) > 1 and head[1].isdigit():
            out.append(int(head[1]))
        else:
            out.append(None)
    return out


# name -> (tensor table, chunk elements)
WORKLOADS = {
    "gpt2_block_768": (lambda: gpt2_block(768), 1 << 22),
    "gpt2_xl": (lambda: gpt2(1600, 48, 6400), 1 << 25),
    "llama_7b": (lambda: llama(4096, 11008, 32), 1 << 26),
    "llama_13b": (lambda: llama(5120, 13824, 40), 1 << 26),
}


def workload(name: str):
    make, chunk_elems = WORKLOADS[name]
    table = make()
    return table, chunk_elems


def total_elems(table) -> int:
    return sum(n for _, n in table)


def n_chunks(table, chunk_elems: int) -> int:
    return -(-total_elems(table) // chunk_elems)
