"""MI355X-native mask-only logits for diffusion-LLM denoising steps (Mosaic, arXiv 2601.06562).

The product is the HIP library behind ``include/mosaic.h``; ``binding`` marshals torch device
tensors to it, ``workloads`` draws the seeded synthetic inputs, ``build`` compiles the library.
"""
from . import binding, workloads  # noqa: F401
from .binding import (MaskOnlyLogits, MosaicError, MosaicPlan, mosaic_compact_scratch_bytes,  # noqa: F401
                      mosaic_mask_compact, mosaic_masked_logits_reduce, mosaic_masked_logits_sample,
                      mosaic_plan_workspace, mosaic_sample_workspace_bytes,
                      mosaic_shift_indices, mosaic_unmask_topn)
