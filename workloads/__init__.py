"""Seeded synthetic inputs shared by the float64 checker and the GPU library (data only, no attention arithmetic)."""
from .batches import AttnDesc, Batch, RemoteShard, build_batch, even_split, synthetic_remote_partials  # noqa: F401
from .configs import FULL, reduced, config1, config2, config3, config3_seed, config4, config5  # noqa: F401
