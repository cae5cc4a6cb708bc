"""The stage workloads: the five benchmark configurations and small test shapes.

Each record fixes the slice of transformer blocks one pipeline stage owns
(Section 4.1, Table 2 give the model family: GPT-style causal decoder and
BERT-style bidirectional encoder with 12h^2+13h parameters per layer) and the
AMDP schedule parameters of Sections 3.1-3.3 (depth d, concurrent pipelines P,
stage index i, injection limit n = 2, accumulation threshold T).
"""
from dataclasses import dataclass, replace

GPT_PRELN_CAUSAL = 0
BERT_POSTLN_BIDIR = 1
FP32 = 0
BF16 = 1


@dataclass(frozen=True)
class StageWorkload:
    name: str
    number: int            # enters the seed
    block_kind: int
    n_layers: int
    d_model: int
    n_heads: int
    d_ffn: int
    seq_len: int
    microbatch: int
    dtype: int
    has_lm_head: bool = False
    vocab: int = 0
    has_embedding: bool = False   # first stage: token + learned position embedding in front of the blocks
    # schedule
    depth: int = 4
    pipelines: int = 2
    stage: int = 1
    inject_limit: int = 2
    threshold: int = 4
    stash_slots: int = 1
    # Adam
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0
    ln_eps: float = 1e-5

    @property
    def tokens(self):
        return self.seq_len * self.microbatch

    @property
    def head_dim(self):
        return self.d_model // self.n_heads

    @property
    def warmup(self):
        return min(self.inject_limit, self.depth - self.stage)

    @property
    def act_slots(self):
        return self.warmup * self.pipelines

    def with_(self, **kw):
        return replace(self, **kw)


CONFIGS = {
    1: StageWorkload("cfg1_gpt_d128_fp32", 1, GPT_PRELN_CAUSAL, 1, 128, 4, 512, 64, 2, FP32,
                     depth=4, pipelines=2, stage=1, threshold=4),
    2: StageWorkload("cfg2_gpt_d1024_bf16", 2, GPT_PRELN_CAUSAL, 4, 1024, 16, 4096, 1024, 4, BF16,
                     depth=6, pipelines=3, stage=3, threshold=8),
    3: StageWorkload("cfg3_bert_d1024_bf16", 3, BERT_POSTLN_BIDIR, 6, 1024, 16, 4096, 512, 8, BF16,
                     depth=4, pipelines=2, stage=1, threshold=8),
    4: StageWorkload("cfg4_gpt_lmhead_d2048_bf16", 4, GPT_PRELN_CAUSAL, 4, 2048, 32, 8192, 2048, 2,
                     BF16, has_lm_head=True, vocab=50257,
                     depth=8, pipelines=3, stage=7, threshold=8),
    5: StageWorkload("cfg5_gpt_d4096_bf16", 5, GPT_PRELN_CAUSAL, 4, 4096, 32, 16384, 2048, 1, BF16,
                     depth=16, pipelines=4, stage=8, threshold=16, stash_slots=3),
}

# Small shapes the CPU oracle finishes in well under a second; dimensions are
# deliberately not multiples of the GPU tile sizes (ragged tails), and the LM
# head vocabulary is odd.
TINY = {
    "gpt": StageWorkload("tiny_gpt", 11, GPT_PRELN_CAUSAL, 2, 16, 2, 40, 8, 2, FP32,
                         depth=4, pipelines=2, stage=0, threshold=4),
    "bert": StageWorkload("tiny_bert", 12, BERT_POSTLN_BIDIR, 2, 16, 2, 40, 8, 2, FP32,
                          depth=4, pipelines=2, stage=1, threshold=4),
    "lmhead": StageWorkload("tiny_lmhead", 13, GPT_PRELN_CAUSAL, 2, 16, 2, 40, 8, 2, FP32,
                            has_lm_head=True, vocab=37,
                            depth=4, pipelines=2, stage=3, threshold=4),
    # first stages: token ids in, small vocabularies so that tokens repeat inside a minibatch
    "embed": StageWorkload("tiny_embed", 26, GPT_PRELN_CAUSAL, 2, 16, 2, 40, 8, 2, FP32, vocab=11,
                           has_embedding=True, depth=4, pipelines=2, stage=0, threshold=4),
    "embed_tile": StageWorkload("tile_embed", 27, GPT_PRELN_CAUSAL, 1, 256, 4, 1024, 256, 2, BF16, vocab=301,
                                has_embedding=True, depth=4, pipelines=2, stage=0, threshold=4),
    "embed_bert_mid": StageWorkload("mid_embed_bert", 28, BERT_POSTLN_BIDIR, 1, 192, 3, 448, 200, 3, BF16, vocab=1031,
                                    has_embedding=True, depth=4, pipelines=2, stage=0, threshold=4),
    # medium shapes: several GPU tiles plus a ragged tail, still seconds on CPU
    "gpt_mid": StageWorkload("mid_gpt", 14, GPT_PRELN_CAUSAL, 2, 192, 3, 448, 200, 2, BF16,
                             depth=6, pipelines=3, stage=2, threshold=6),
    "bert_mid": StageWorkload("mid_bert", 15, BERT_POSTLN_BIDIR, 2, 192, 3, 448, 200, 3, BF16,
                              depth=4, pipelines=2, stage=1, threshold=4),
    "lmhead_mid": StageWorkload("mid_lmhead", 16, GPT_PRELN_CAUSAL, 1, 192, 3, 448, 136, 2, BF16,
                                has_lm_head=True, vocab=1031,
                                depth=4, pipelines=2, stage=3, threshold=4),
    # tile-aligned shapes that take the MFMA kernels
    "gpt_tile": StageWorkload("tile_gpt", 17, GPT_PRELN_CAUSAL, 2, 256, 4, 1024, 256, 2, BF16,
                              depth=6, pipelines=3, stage=3, threshold=6),
    "bert_tile": StageWorkload("tile_bert", 18, BERT_POSTLN_BIDIR, 2, 256, 4, 1024, 256, 2, BF16,
                               depth=4, pipelines=2, stage=1, threshold=4),
    # head dimension 128, two key blocks per query block
    "gpt_tile128": StageWorkload("tile_gpt_dh128", 20, GPT_PRELN_CAUSAL, 1, 256, 2, 512, 256, 2, BF16,
                                 depth=4, pipelines=2, stage=1, threshold=4),
    "bert_tile128": StageWorkload("tile_bert_dh128", 21, BERT_POSTLN_BIDIR, 1, 256, 2, 512, 384, 2, BF16,
                                  depth=4, pipelines=2, stage=1, threshold=4),
    # multiples of 64 but not of 128: the 64-row matrix tiles
    "gpt_tile64": StageWorkload("tile64_gpt", 22, GPT_PRELN_CAUSAL, 2, 192, 3, 768, 128, 2, BF16,
                                depth=4, pipelines=2, stage=1, threshold=4),
    # every ragged last tile the 128- and 256-wide GEMM tiles can meet: widths 320 = 256 + 64,
    # 640 = 2*256 + 128, 960 = 3*256 + 192; 384 tokens = 256 + 128
    "gpt_tile_edge": StageWorkload("tile_edge_gpt", 29, GPT_PRELN_CAUSAL, 2, 320, 5, 640, 128, 3, BF16,
                                   depth=4, pipelines=2, stage=1, threshold=4),
    # head dimension 50 (the paper's BERT-style width / heads): no fused attention, unaligned heads
    "bert_dh50": StageWorkload("tiny_bert_dh50", 23, BERT_POSTLN_BIDIR, 1, 400, 8, 800, 24, 2, BF16,
                               depth=4, pipelines=2, stage=1, threshold=4),
    # head dimensions the fused attention reaches by zero-padding (50 -> 64, 96 -> 128)
    "bert_tile_dh50": StageWorkload("tile_bert_dh50", 24, BERT_POSTLN_BIDIR, 1, 400, 8, 800, 128, 2, BF16,
                                    depth=4, pipelines=2, stage=1, threshold=4),
    "gpt_tile_dh96": StageWorkload("tile_gpt_dh96", 25, GPT_PRELN_CAUSAL, 1, 192, 2, 384, 256, 1, BF16,
                                   depth=4, pipelines=2, stage=1, threshold=4),
    "lmhead_tile": StageWorkload("tile_lmhead", 19, GPT_PRELN_CAUSAL, 1, 256, 4, 1024, 256, 2, BF16,
                                 has_lm_head=True, vocab=1931,
                                 depth=4, pipelines=2, stage=3, threshold=4),
}


# Stages shaped like the paper's own models (Table 2: hidden 1600; 25 heads for
# the GPT-style model, 32 for the BERT-style one; sequence 1024, microbatch 4;
# 48 layers over a depth-8 pipeline = 6 layers per stage).
PAPER = {
    "paper_gpt_h1600": StageWorkload("paper_gpt_h1600_bf16", 31, GPT_PRELN_CAUSAL, 6, 1600, 25, 6400, 1024, 4, BF16,
                                     depth=8, pipelines=4, stage=4, threshold=8),
    "paper_bert_h1600": StageWorkload("paper_bert_h1600_bf16", 32, BERT_POSTLN_BIDIR, 6, 1600, 32, 6400, 1024, 4, BF16,
                                      depth=8, pipelines=4, stage=4, threshold=8),
}


# First stage of configuration 2's model: token ids in, GPT-2's vocabulary.
FIRST = {
    "first_gpt_d1024": StageWorkload("first_gpt_d1024_bf16", 33, GPT_PRELN_CAUSAL, 4, 1024, 16, 4096, 1024, 4, BF16,
                                     vocab=50257, has_embedding=True, depth=6, pipelines=3, stage=0, threshold=8),
}


def get(key):
    if isinstance(key, int):
        return CONFIGS[key]
    if key in TINY:
        return TINY[key]
    if key in PAPER:
        return PAPER[key]
    if key in FIRST:
        return FIRST[key]
    if key.isdigit():
        return CONFIGS[int(key)]
    for c in CONFIGS.values():
        if c.name == key:
            return c
    raise KeyError(key)
