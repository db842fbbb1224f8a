"""MI355X-native hot path of Harli (arXiv 2511.11729): decode step + LoRA finetune unit
over one unified HBM pool, behind the C ABI declared in include/harli.h."""
from . import binding  # noqa: F401
from .binding import Pool, Context, HarliError, lib  # noqa: F401
