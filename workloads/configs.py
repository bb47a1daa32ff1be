"""The synthetic workloads (shapes follow the paper's: 16x VQ grids of
256-4096 tokens, whole-row draft blocks, a prefilled conditioning prefix, a
LlamaGen-class decoder; supplement "Primer on Tar").  Data only: no arithmetic
of the method lives here.
"""
import copy

_MODELS = {
    "tiny": dict(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024,
                 dtype="f32", rms_eps=1e-5),
    "small": dict(n_layers=8, d_model=1024, n_heads=16, head_dim=64, d_ffn=2816, vocab=8192,
                  dtype="bf16", rms_eps=1e-5),
    "7b": dict(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008, vocab=16384,
               dtype="bf16", rms_eps=1e-5),
}

# h, w: drafter grid; r: linear ratio; L: draft block (whole rows of the target grid);
# radius/expand: local expansion; sigma: draft-logit noise std (None: draft logits ~ N(0, 2)).
CONFIGS = {
    "cfg1": dict(model="tiny", prefix=32, h=8, w=8, r=2, L=256, B=1, radius=1, expand=1,
                 sigma=None, draft_std=2.0, seed=0),
    "cfg2": dict(model="small", prefix=64, h=16, w=16, r=2, L=256, B=4, radius=1, expand=1,
                 sigma=None, draft_std=2.0, seed=0),
    "cfg3": dict(model="7b", prefix=128, h=24, w=24, r=2, L=576, B=1, radius=1, expand=1,
                 sigma=1.0, seed=0),
    "cfg4": dict(model="7b", prefix=128, h=32, w=32, r=2, L=1024, B=4, radius=2, expand=1,
                 sigma=1.0, seed=0),
    "cfg5_L256": dict(model="7b", prefix=128, h=32, w=32, r=2, L=256, B=16, radius=1, expand=1,
                      sigma=1.0, seed=0),
    "cfg5_L512": dict(model="7b", prefix=128, h=32, w=32, r=2, L=512, B=16, radius=1, expand=1,
                      sigma=1.0, seed=0),
    "cfg5_L1024": dict(model="7b", prefix=128, h=32, w=32, r=2, L=1024, B=16, radius=1, expand=1,
                       sigma=1.0, seed=0),
    # the paper's best setting (Sec. 4, ratio 4: a 16x16 draft of the 64x64 grid; radius 3): data-only variants
    "cfg1_r4": dict(model="tiny", prefix=32, h=4, w=4, r=4, L=256, B=2, radius=3, expand=1,
                    sigma=None, draft_std=2.0, seed=0),
    "cfg4_r4": dict(model="7b", prefix=128, h=16, w=16, r=4, L=1024, B=4, radius=3, expand=1,
                    sigma=1.0, seed=0),
}


def get(name):
    """Config `name` with the model dims merged in and derived sizes added."""
    c = copy.deepcopy(CONFIGS[name])
    c["name"] = name
    c["model_name"] = c["model"]
    c["model"] = copy.deepcopy(_MODELS[c["model"]])
    c["H"], c["W"] = c["r"] * c["h"], c["r"] * c["w"]
    c["T"] = c["H"] * c["W"]                       # image tokens
    c["max_seq"] = c["prefix"] + c["T"]
    assert c["L"] % c["W"] == 0 and c["T"] % c["L"] == 0
    return c


def model(name):
    return copy.deepcopy(_MODELS[name])
