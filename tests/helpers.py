"""Small model shapes of the three families, for tests that run the oracle in seconds."""
import ppd_inputs as pi


def small_cfg(family: str, **kw) -> pi.ModelConfig:
    base = {
        # same family switches as the benchmark configs, shrunk; widths chosen to be ragged
        "tiny": pi.CONFIGS["tiny"],
        "opt": pi.CONFIGS["opt125m"].replace(name="opt_small", n_layers=4, d_model=192, n_heads=3, d_ff=520,
                                             vocab=1531, max_ctx=96, n_prompt=12, n_gen=20, exit_layer=2),
        "llama": pi.CONFIGS["llama7b"].replace(name="llama_small", n_layers=6, d_model=256, n_heads=2,
                                               d_ff=696, vocab=1237, max_ctx=96, n_prompt=12, n_gen=20,
                                               exit_layer=3),
    }[family]
    return base.replace(**kw) if kw else base
