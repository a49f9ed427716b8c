"""MI355X-native trimmed-LM-head path of VocabTrim: count -> select/gather -> draft step.

The arithmetic lives in libvocabtrim.so (hand-written HIP for gfx950, C ABI in
include/vocabtrim.h); this package is the thin binding plus the seeded input
generators used by tests and the benchmark.
"""
from .binding import (MultiStepWorkspace, StepWorkspace, VocabTrimError, build_trimmed_head, build_trimmed_heads,
                      choose_k, count_tokens, draft_head_step, draft_head_step_multi, draft_head_step_multi_plan, draft_head_step_plan, draft_head_step_static,
                      draft_tree_level, load_library, tree_expand, tree_rerank)

__all__ = ["MultiStepWorkspace", "StepWorkspace", "VocabTrimError", "build_trimmed_head", "build_trimmed_heads",
           "choose_k", "count_tokens", "draft_head_step", "draft_head_step_multi", "draft_head_step_multi_plan", "draft_head_step_plan",
           "draft_head_step_static", "draft_tree_level", "load_library", "tree_expand", "tree_rerank"]
