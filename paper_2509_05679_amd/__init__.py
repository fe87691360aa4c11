"""MI355X-native decoupled data-parallel training step (libdds) and its binding."""
from .binding import (DdsError, Spec, Trainer, dds_arena_bytes, dds_schedule, lib, EXPORTS,  # noqa: F401
                      DDS_OK, DDS_EINVAL, DDS_ENOMEM, DDS_EHIP, DDS_EUNSUPPORTED)
