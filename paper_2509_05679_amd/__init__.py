"""MI355X-native decoupled data-parallel training step (libdds) and its binding."""
from .binding import (DdsError, Spec, Trainer, dds_arena_bytes, dds_schedule, dds_step_size, lib, EXPORTS,  # noqa: F401
                      DDS_OK, DDS_EINVAL, DDS_ENOMEM, DDS_EHIP, DDS_EUNSUPPORTED,
                      DDS_ETA_CONSTANT, DDS_ETA_PIECEWISE, DDS_ETA_DIMINISHING,
                      DDS_DBG_INPUT, DDS_DBG_OUTPUT, DDS_DBG_ERROR, DDS_DBG_LABELS, DDS_DBG_SNAPSHOT)
