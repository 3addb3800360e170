"""The five synthetic workloads (model shapes, batch, KV lengths, tree shapes) and the B = 8 bench point.

Pure data: no arithmetic of the method lives here.  Both the CPU oracle's tests and the HIP path's tests
read these; neither side imports the other.
"""

TINY = dict(name="tiny", n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=704, vocab=1024,
            rms_eps=1e-6, rope_theta=10000.0, dtype="fp32")
Q1P5B = dict(name="1.5b", n_layers=28, d_model=1536, n_q_heads=12, n_kv_heads=2, head_dim=128, d_ffn=8960,
             vocab=151936, rms_eps=1e-6, rope_theta=10000.0, dtype="bf16")
Q7B = dict(name="7b", n_layers=28, d_model=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, d_ffn=18944,
           vocab=152064, rms_eps=1e-6, rope_theta=10000.0, dtype="bf16")


def draft_of(model):
    """The 1-layer draft head of the same width as its target."""
    d = dict(model)
    d["n_layers"] = 1
    d["name"] = model["name"] + "-draft"
    return d


def with_dtype(model, dtype):
    """The same model computed in another arithmetic type ("bf16", "fp16" or "fp32")."""
    d = dict(model)
    d["dtype"] = dtype
    return d


def scaled(model, n_layers):
    """The same layer geometry with fewer layers (for parity cases the CPU oracle finishes quickly)."""
    d = dict(model)
    d["n_layers"] = n_layers
    d["name"] = f"{model['name']}-L{n_layers}"
    return d


# tree: ("chain", depth) or ("tree", top_k, depth, n_nodes); N counts the root.
CONFIGS = {
    "cfg1": dict(model=TINY, B=8, group=4, prompt_len=32, kv_lo=32, kv_hi=32, tree=("chain", 4), N=5,
                 accept="greedy", plant_p=None, new_tokens=64, page_size=16, seed=0),
    "cfg2": dict(model=Q1P5B, B=16, group=8, prompt_len=128, kv_lo=512, kv_hi=512, tree=("chain", 5), N=6,
                 accept="greedy", plant_p=0.7, page_size=16, seed=0),
    "cfg3": dict(model=Q7B, B=64, group=8, prompt_len=256, kv_lo=256, kv_hi=2048, tree=("tree", 4, 5, 24), N=24,
                 accept="greedy", plant_p=0.7, page_size=16, seed=0),
    "cfg4": dict(model=Q7B, B=256, group=8, prompt_len=256, kv_lo=1024, kv_hi=4096, tree=("plan", (1, 2, 4, 8)),
                 N=8, accept="greedy", plant_p=0.6, page_size=16, seed=0),
    "cfg5": dict(model=Q7B, B=128, group=8, prompt_len=256, kv_lo=256, kv_hi=3072, tree=("tree", 4, 6, 32), N=32,
                 accept="reject", temperature=1.0, plant_p=0.65, page_size=16, seed=0),
    # low end of the metric's B = 8..256 range: one prompt x group 8
    "b8": dict(model=Q7B, B=8, group=8, prompt_len=256, kv_lo=256, kv_hi=2048, tree=("plan", (1, 6, 24)), N=24,
               accept="greedy", plant_p=0.7, page_size=16, seed=0),
}

# defaults of the concurrency rule's free constants (the paper prints no values)
PLAN_DEFAULTS = dict(alpha=0.5, K_max=4, L_max=6, N_cap=64)
