"""MI355X-native edge-side verification round of WISV (hand-written HIP behind a C ABI).

`binding` wraps libwisv.so (build it with `python -m paper_2604_17701_amd.build`).
Nothing here computes on the CPU; without the built library and a GPU the calls raise.
"""
from . import binding  # noqa: F401
from .binding import (Context, DeviceRound, WisvError, wisv_ctx_create, wisv_destroy,  # noqa: F401
                      wisv_verify_round)
