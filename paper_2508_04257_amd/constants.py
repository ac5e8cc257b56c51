"""Per-model constants of the stable outliers (paper, Appendix D table): the emergence-stage
layer l_E whose output is scanned once per prefill, and the channels the extreme activations
sit in.  These are inputs of ``kvs_predict_sinks`` (which layer's hidden state to pass, which
channels to scan); identifying them needs model weights and is not part of the library."""

MODEL_TABLE = {
    # name: (layers, l_E, hidden size, outlier channels)
    "LLaMA2-7B": (32, 1, 4096, (2533, 1415)),
    "LLaMA2-13B": (40, 3, 5120, (4743, 2100)),
    "Mistral-7B": (32, 1, 4096, (2070, 3398)),
    "LLaMA3-8B": (32, 1, 4096, (788, 1384, 4062)),
    "LLaMA3.1-8B-instruct": (32, 1, 4096, (788, 1384, 4062)),
    "LLaMA3.2-1B": (16, 1, 2048, (400, 698, 2029, 1159)),
    "LLaMA3.2-3B": (28, 1, 3072, (588, 1016, 3046, 1731)),
}
