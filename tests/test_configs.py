"""The workload configurations against what the paper prints about its layers
(tests/golden/paper_attention_layers.txt) and against its cost model."""
import os

from inputs.fields import CONFIGS

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden",
                      "paper_attention_layers.txt")


def read_layers():
    rows = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        name, *vals = line.split()
        rows[name] = dict(zip(("nside", "pixels", "dim", "heads", "n", "b", "local", "gqa"),
                              map(int, vals)))
    return rows


def test_paper_layer_configurations_match_the_architecture_table():
    layers = read_layers()
    assert set(layers) == {"stage1", "stage2", "bottleneck"}
    for cid, name in ((10, "stage1"), (11, "stage2"), (12, "bottleneck")):
        cfg, row = CONFIGS[cid], layers[name]
        assert row["pixels"] == 12 * row["nside"] ** 2          # the HEALPix pixel count
        assert cfg.n_tokens == row["pixels"]
        assert cfg.heads == row["heads"] and cfg.head_dim * cfg.heads == row["dim"]
        assert cfg.block_tokens == row["b"] and cfg.n_select == row["n"]
        assert cfg.kv_heads * row["gqa"] == cfg.heads
        assert cfg.block_h == 1                                   # blocks of consecutive tokens
        # a large local block is a whole number of sparse blocks, and they tile the layer
        assert row["local"] % row["b"] == 0 and cfg.n_blocks % (row["local"] // row["b"]) == 0


def test_flop_count_is_the_selection_and_local_terms_of_the_cost_model():
    """Cost model of the Block-Sparse Attention subsection: N n b (selection) +
    N b (local) token pairs, each a D-long dot product for the scores and a
    D-long update for the output (2 flop per multiply-add)."""
    for cfg in CONFIGS.values():
        pairs = cfg.n_tokens * cfg.n_select * cfg.block_tokens + cfg.n_tokens * cfg.block_tokens
        assert cfg.fwd_flops() == cfg.batch * cfg.heads * pairs * cfg.head_dim * 2 * 2
