"""MI355X rollout generation: thin ctypes binding over librollout.so (argument marshalling
only; every step of the path runs in the library's HIP kernels)."""
from .binding import (LIB_PATH, Rollout, RolloutError, load_library, model_desc_from_shape,  # noqa: F401
                      rollout_philox_words, rollout_plan_pages, rollout_policy_loss, rollout_sample,
                      rollout_sample_static, PagePool)
