"""MI355X-native verification pass with early exits (speculative edge-cloud
decoding, server side).  The work is done by libeeverify.so (HIP, gfx950);
this package is its ctypes binding and build script."""
from .binding import (EEError, Model, Session, VerifyOutput, ee_verify_batch, ee_verify_sampled_batch, ee_debug_mfma_layout, ee_debug_div_small, ee_tune_k_split, ee_device_synchronize, ee_debug_copy, ee_latency_model,
                      load_library, lib_path, EXPORTS, HOLD_LAST, KEEP_LOGITS, NO_AUTOCOMMIT, SAMPLING,
                      TIME_LAUNCHES, OPT_ATT_SPLITS, OPT_SCATTER_PAGES, OPT_HEAD_BATCH, LAUNCH_NAMES, EE_OK, EE_NOT_READY, EE_DONE, EE_EINVAL, EE_ESTATE, EE_ECAPACITY, EE_EIO,
                      EE_EFORMAT, EE_EDEVICE, EE_MAX_M, EE_MAX_EXITS, EE_MAX_BATCH, EE_MAX_ROWS)
