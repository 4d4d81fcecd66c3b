"""Shapes and layouts used by the tests (pure data, no arithmetic of the method)."""
from oracle.reshard_oracle import GenLayout, Model, TrainLayout

# The five BASELINE configurations (index = config number - 1).
BASELINE = [
    dict(name="tiny", model=Model(2, 256, 4, 4, 64, 688, 1024), train=TrainLayout(1, 4, 1), gen=GenLayout(1, 2),
         mat="all"),
    dict(name="llama7b", model=Model(32, 4096, 32, 32, 128, 11008, 32000), train=TrainLayout(1, 8, 1),
         gen=GenLayout(1, 2), mat="all"),
    dict(name="llama13b", model=Model(40, 5120, 40, 40, 128, 13824, 32000), train=TrainLayout(2, 4, 1),
         gen=GenLayout(1, 2), mat="all"),
    dict(name="llama34b_gqa", model=Model(48, 8192, 64, 8, 128, 22016, 32000), train=TrainLayout(2, 8, 1),
         gen=GenLayout(1, 4), mat=[0, 2, 4, 6]),
    dict(name="llama70b_gqa", model=Model(80, 8192, 64, 8, 128, 28672, 128256), train=TrainLayout(4, 8, 1),
         gen=GenLayout(1, 4), mat=[0, 31]),
]

# Small shapes the oracle (and the pure-Python brute force) finishes in seconds.  They
# cover MHA and GQA, rows that are only 2/4/8-byte aligned, padding between tensors
# (hidden*2 not a multiple of 256), merged pipeline stages, p_g > 1 and d > 1.
SMALL = [
    dict(name="mha_tp4_tp2", model=Model(2, 32, 4, 4, 8, 24, 64), train=TrainLayout(1, 4, 1), gen=GenLayout(1, 2)),
    dict(name="gqa_tp4_tp1", model=Model(2, 48, 8, 4, 4, 20, 32), train=TrainLayout(1, 4, 1), gen=GenLayout(1, 1)),
    dict(name="gqa_tp2pp2_tp1", model=Model(4, 40, 8, 2, 8, 18, 16), train=TrainLayout(2, 2, 1), gen=GenLayout(1, 1)),
    dict(name="gqa_tp4pp4_tp2pp2", model=Model(4, 24, 8, 4, 4, 28, 32), train=TrainLayout(4, 4, 1), gen=GenLayout(2, 2)),
    dict(name="mha_dp2", model=Model(2, 16, 4, 4, 4, 12, 16), train=TrainLayout(2, 2, 2), gen=GenLayout(1, 1)),
    dict(name="odd_rows", model=Model(1, 6, 2, 2, 3, 10, 8), train=TrainLayout(1, 2, 1), gen=GenLayout(1, 1)),
    dict(name="same_layout", model=Model(2, 32, 4, 2, 8, 24, 64), train=TrainLayout(2, 2, 1), gen=GenLayout(2, 2)),
    # eight pipeline stages merged into one, TP unchanged (micro-DP 8 from PP alone): the layout of Section 8.4's 70B example
    dict(name="pp8_merge_tp2", model=Model(8, 16, 4, 2, 4, 12, 16), train=TrainLayout(8, 2, 1), gen=GenLayout(1, 2)),
]

# Medium shapes: tens of MB, several 128 KiB tiles per descriptor with ragged tails,
# rows that are 16-, 8-, 4- and only 2-byte aligned, GQA, merged pipeline stages.
MEDIUM = [
    dict(name="mid_gqa_tp8pp2_tp2", model=Model(4, 512, 16, 8, 32, 2760, 2000), train=TrainLayout(2, 8, 1),
         gen=GenLayout(1, 2)),
    dict(name="mid_mha_tp4_tp1", model=Model(3, 768, 12, 12, 64, 2052, 5004), train=TrainLayout(1, 4, 1),
         gen=GenLayout(1, 1)),
    dict(name="mid_gqa_tp4pp4_tp2pp2_dp2", model=Model(8, 520, 8, 4, 65, 1404, 1000), train=TrainLayout(4, 4, 2),
         gen=GenLayout(2, 2)),
]
